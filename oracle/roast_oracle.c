/*
 * ROAST hashing -- plain CPU oracle (TEST INFRASTRUCTURE ONLY).
 *
 * This file is the slow, obviously-correct statement of what the ROAST hot
 * path computes.  It exists so that the HIP kernels can be checked against
 * something written straight from the paper.  It is not part of the product:
 * only the tests, the smoke check and the cpu_baseline leg of the benchmark
 * may call it, and it shares no code, header, table or helper with the HIP
 * library.  Everything floating point is done in double.
 *
 * What each function follows (arXiv 2207.10702):
 *   - oracle_locate           : the hash maps h1 / h2 (Section 4.1, "Lookup"
 *                               and "Matrix multiplication" paragraphs) and
 *                               the sign map g (end of Section 4.1).  The
 *                               paper only asks for a universal hash
 *                               function; the family used here is the
 *                               Carter-Wegman multiply-add-mod-prime family,
 *                               ((c0*k0 + c1*k1 + c2*k2 + c3) mod P) mod range.
 *   - oracle_elem_sign        : the per-element reading of the sign map g
 *                               (use_sign == 2; the theory of Section 5
 *                               writes g(i) per parameter), same hash family,
 *                               keyed by the element's coordinates.
 *   - oracle_element_index    : the ROAST-MM mapping equation of Section 4.1,
 *                               W[i,j] = lambda * M[h2(C1,C2) + Z2*O1 + O2].
 *   - oracle_materialize_w    : that equation, evaluated element by element.
 *   - oracle_gemm_nn          : the result Algorithm 1 ensures, Y = X * W.
 *   - oracle_gemm_nt / _tn    : dX = dY * W^T and dW = X^T * dY, the ordinary
 *                               matrix-product gradients (Section 4.3).
 *   - oracle_scatter_dm       : the gradient equation of Section 4.3 /
 *                               Appendix A.1: grad M[i] is the lambda-scaled
 *                               sum of the gradients of every recovered
 *                               parameter that maps to slot i (the sign g is
 *                               included, as the chain rule requires).
 *   - oracle_dm_window        : the same sum restricted to a window of slots,
 *                               so that big problems can be checked slot by
 *                               slot without forming all of dW.
 *   - oracle_embed_fwd / _bwd : the lookup equation of Section 4.1,
 *                               w[i] = lambda * M[h1(C(i)) + O(i)], and its
 *                               gradient by the same Section 4.3 sum.
 *
 * Parity pins for every function above are in tests/test_oracle_pins.py
 * (closed forms, library GEMM on the identity-hash special case, finite
 * differences, adjoint identities, the variance formula of Theorem 1).
 * The paper prints no worked numeric example (Figure 1 is an image), so the
 * particular hash constants are pinned only by this definition.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* Threads the OpenMP loops below really get (reported next to the oracle's timing; no arithmetic). */
int oracle_num_threads(void) {
  int n = 1;
#ifdef _OPENMP
#pragma omp parallel
  {
#pragma omp single
    n = omp_get_num_threads();
  }
#endif
  return n;
}

typedef struct {
  uint64_t P;              /* prime modulus, 2 <= P < 2^32                      */
  uint64_t a0, a1, a2, a3; /* offset hash coefficients, all < P                 */
  uint64_t s0, s1, s2, s3; /* sign hash coefficients, all < P                   */
  uint32_t use_sign;       /* 0: sign is +1 everywhere; 1: one sign per block    */
                           /* (tile / chunk); 2: one sign per element            */
  uint32_t align;          /* offsets are multiples of align (1 = the paper)    */
} oracle_hash_t;

/* Carter-Wegman value of a 3-part key.  Keys are reduced mod P first and every
 * product is reduced before the sum, so nothing exceeds 64 bits. */
static uint64_t cw_value(uint64_t P, uint64_t c0, uint64_t c1, uint64_t c2, uint64_t c3,
                         uint64_t k0, uint64_t k1, uint64_t k2) {
  uint64_t t0 = (c0 * (k0 % P)) % P;
  uint64_t t1 = (c1 * (k1 % P)) % P;
  uint64_t t2 = (c2 * (k2 % P)) % P;
  return (t0 + t1 + t2 + c3) % P;
}

/* Offset and sign of the block (tile or chunk) with key (k0,k1,k2).
 * The block has `len` scalars and must fit: offsets range over
 * {0, ..., m_size - len} (inclusive), restricted to multiples of align.
 * Returns 0 on success, 1 if the block cannot fit. */
int oracle_locate(const oracle_hash_t* h, uint64_t k0, uint64_t k1, uint64_t k2,
                  int64_t m_size, int64_t len, int64_t* off, int32_t* sgn) {
  if (len <= 0 || m_size < len || h->align == 0 || h->P < 2) return 1;
  uint64_t nslots = (uint64_t)(m_size - len) / h->align + 1;
  uint64_t u = cw_value(h->P, h->a0, h->a1, h->a2, h->a3, k0, k1, k2);
  *off = (int64_t)(h->align * (u % nslots));
  if (h->use_sign == 1) {
    uint64_t v = cw_value(h->P, h->s0, h->s1, h->s2, h->s3, k0, k1, k2);
    *sgn = 1 - 2 * (int32_t)(v & 1u);
  } else {
    *sgn = 1;   /* no sign, or the sign belongs to the element (oracle_elem_sign) */
  }
  return 0;
}

/* Per-element variant of the sign map g (use_sign == 2): the same sign hash, keyed by the
 * element's own coordinates -- (layer, i, j) for W[i,j], (table, row, i) for element i of a looked
 * up row -- instead of the block's.  +1 in the other modes. */
int32_t oracle_elem_sign(const oracle_hash_t* h, uint64_t k0, uint64_t k1, uint64_t k2) {
  if (h->use_sign != 2) return 1;
  uint64_t v = cw_value(h->P, h->s0, h->s1, h->s2, h->s3, k0, k1, k2);
  return 1 - 2 * (int32_t)(v & 1u);
}

/* Tile grid of one ROAST-MM layer: ceil(H/Z1) x ceil(O/Z2) tiles, row-major in
 * (x, y) with x along H.  Key = (layer, x, y). */
int oracle_tile_index(const oracle_hash_t* h, uint32_t layer, int64_t H, int64_t O,
                      int32_t Z1, int32_t Z2, int64_t m_size, int64_t* off, int8_t* sgn) {
  if (H <= 0 || O <= 0 || Z1 <= 0 || Z2 <= 0) return 1;
  int64_t ntx = (H + Z1 - 1) / Z1, nty = (O + Z2 - 1) / Z2;
  for (int64_t x = 0; x < ntx; ++x)
    for (int64_t y = 0; y < nty; ++y) {
      int64_t o; int32_t s;
      if (oracle_locate(h, layer, (uint64_t)x, (uint64_t)y, m_size, (int64_t)Z1 * Z2, &o, &s)) return 1;
      off[x * nty + y] = o;
      sgn[x * nty + y] = (int8_t)s;
    }
  return 0;
}

/* Slot of M and sign used by the virtual weight W[i,j]. */
int oracle_element_index(const oracle_hash_t* h, uint32_t layer, int32_t Z1, int32_t Z2,
                         int64_t m_size, int64_t i, int64_t j, int64_t* idx, int32_t* sgn) {
  int64_t c1 = i / Z1, c2 = j / Z2;   /* tile coordinates      */
  int64_t o1 = i % Z1, o2 = j % Z2;   /* offsets inside a tile */
  int64_t base;
  if (oracle_locate(h, layer, (uint64_t)c1, (uint64_t)c2, m_size, (int64_t)Z1 * Z2, &base, sgn)) return 1;
  *idx = base + (int64_t)Z2 * o1 + o2;
  *sgn *= oracle_elem_sign(h, layer, (uint64_t)i, (uint64_t)j);
  return 0;
}

/* Round a double to the nearest bfloat16 (ties to even) and return it as a
 * double.  Only finite, float-representable inputs are used here. */
double oracle_round_bf16(double v) {
  float f = (float)v;
  uint32_t u;
  memcpy(&u, &f, 4);
  uint32_t keep = u >> 16, rest = u & 0xFFFFu;
  if (rest > 0x8000u || (rest == 0x8000u && (keep & 1u))) keep += 1;
  u = keep << 16;
  memcpy(&f, &u, 4);
  return (double)f;
}

/* W[i*O + j] for the whole H x O virtual matrix, one element at a time.
 * round_bf16 != 0 rounds sign*M to bfloat16 before the lambda scale: this is
 * the "as computed" reference for the bf16 path, where the weight operand is
 * held in bfloat16 and lambda is applied to the accumulated result. */
int oracle_materialize_w(const oracle_hash_t* h, uint32_t layer, int64_t H, int64_t O,
                         int32_t Z1, int32_t Z2, int64_t m_size, double lambda,
                         const float* M, int32_t round_bf16, double* W) {
  for (int64_t i = 0; i < H; ++i)
    for (int64_t j = 0; j < O; ++j) {
      int64_t idx; int32_t s;
      if (oracle_element_index(h, layer, Z1, Z2, m_size, i, j, &idx, &s)) return 1;
      double v = (double)s * (double)M[idx];
      if (round_bf16) v = oracle_round_bf16(v);
      W[i * O + j] = lambda * v;
    }
  return 0;
}

/* Y[I x O] = X[I x H] * W[H x O] */
void oracle_gemm_nn(int64_t I, int64_t H, int64_t O, const double* X, const double* W, double* Y) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < I; ++i) {
    double* y = Y + i * O;
    for (int64_t o = 0; o < O; ++o) y[o] = 0.0;
    for (int64_t k = 0; k < H; ++k) {
      double x = X[i * H + k];
      const double* w = W + k * O;
      for (int64_t o = 0; o < O; ++o) y[o] += x * w[o];
    }
  }
}

/* dX[I x H] = dY[I x O] * W^T */
void oracle_gemm_nt(int64_t I, int64_t H, int64_t O, const double* dY, const double* W, double* dX) {
#pragma omp parallel for schedule(static)
  for (int64_t i = 0; i < I; ++i)
    for (int64_t k = 0; k < H; ++k) {
      double acc = 0.0;
      const double* w = W + k * O;
      const double* g = dY + i * O;
      for (int64_t o = 0; o < O; ++o) acc += g[o] * w[o];
      dX[i * H + k] = acc;
    }
}

/* dW[H x O] = X^T * dY */
void oracle_gemm_tn(int64_t I, int64_t H, int64_t O, const double* X, const double* dY, double* dW) {
#pragma omp parallel for schedule(static)
  for (int64_t k = 0; k < H; ++k) {
    double* w = dW + k * O;
    for (int64_t o = 0; o < O; ++o) w[o] = 0.0;
    for (int64_t i = 0; i < I; ++i) {
      double x = X[i * H + k];
      const double* g = dY + i * O;
      for (int64_t o = 0; o < O; ++o) w[o] += x * g[o];
    }
  }
}

/* dM[slot(i,j)] += lambda * sign(i,j) * dW[i,j] for every virtual weight. */
int oracle_scatter_dm(const oracle_hash_t* h, uint32_t layer, int64_t H, int64_t O,
                      int32_t Z1, int32_t Z2, int64_t m_size, double lambda,
                      const double* dW, double* dM) {
  for (int64_t i = 0; i < H; ++i)
    for (int64_t j = 0; j < O; ++j) {
      int64_t idx; int32_t s;
      if (oracle_element_index(h, layer, Z1, Z2, m_size, i, j, &idx, &s)) return 1;
      dM[idx] += lambda * (double)s * dW[i * O + j];
    }
  return 0;
}

/* The same gradient for slots j0 <= slot < j1 only: every virtual weight is
 * visited, and those landing in the window get their full dW[i,j] (a sum over
 * all I rows) computed on the spot.  win[slot - j0] is accumulated into. */
int oracle_dm_window(const oracle_hash_t* h, uint32_t layer, int64_t I, int64_t H, int64_t O,
                     int32_t Z1, int32_t Z2, int64_t m_size, double lambda,
                     const double* X, const double* dY, int64_t j0, int64_t j1, double* win) {
  int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t i = 0; i < H; ++i) {
    for (int64_t j = 0; j < O; ++j) {
      int64_t idx; int32_t s;
      if (oracle_element_index(h, layer, Z1, Z2, m_size, i, j, &idx, &s)) { err = 1; continue; }
      if (idx < j0 || idx >= j1) continue;
      double acc = 0.0;
      for (int64_t r = 0; r < I; ++r) acc += X[r * H + i] * dY[r * O + j];
      double add = lambda * (double)s * acc;
#pragma omp atomic
      win[idx - j0] += add;
    }
  }
  return err;
}

/* out[n, i] = lambda * g * M[h1(chunk) + (i mod Z)], chunk key = (table, row, i div Z).
 * The chunk's offset and sign are found once per chunk, then its elements are copied one by one. */
int oracle_embed_fwd(const oracle_hash_t* h, int64_t D, int32_t Z, int64_t m_size, double lambda,
                     int64_t N, const int64_t* rows, const uint32_t* tables,
                     const float* M, double* out) {
  for (int64_t n = 0; n < N; ++n) {
    if (rows[n] < 0) return 1;
    for (int64_t c = 0; c * Z < D; ++c) {
      int64_t base; int32_t s;
      if (oracle_locate(h, tables[n], (uint64_t)rows[n], (uint64_t)c, m_size, Z, &base, &s)) return 1;
      for (int64_t i = c * Z; i < D && i < (c + 1) * Z; ++i) {
        int32_t g = s * oracle_elem_sign(h, tables[n], (uint64_t)rows[n], (uint64_t)i);
        out[n * D + i] = lambda * (double)g * (double)M[base + i % Z];
      }
    }
  }
  return 0;
}

/* dM[h1(chunk) + (i mod Z)] += lambda * g * dOut[n, i] */
int oracle_embed_bwd(const oracle_hash_t* h, int64_t D, int32_t Z, int64_t m_size, double lambda,
                     int64_t N, const int64_t* rows, const uint32_t* tables,
                     const double* dOut, double* dM) {
  for (int64_t n = 0; n < N; ++n) {
    if (rows[n] < 0) return 1;
    for (int64_t c = 0; c * Z < D; ++c) {
      int64_t base; int32_t s;
      if (oracle_locate(h, tables[n], (uint64_t)rows[n], (uint64_t)c, m_size, Z, &base, &s)) return 1;
      for (int64_t i = c * Z; i < D && i < (c + 1) * Z; ++i) {
        int32_t g = s * oracle_elem_sign(h, tables[n], (uint64_t)rows[n], (uint64_t)i);
        dM[base + i % Z] += lambda * (double)g * dOut[n * D + i];
      }
    }
  }
  return 0;
}
