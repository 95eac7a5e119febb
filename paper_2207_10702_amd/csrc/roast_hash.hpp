// Integer side of ROAST: block key -> (offset in M, sign).  Host and device share this one
// implementation inside the library (the CPU oracle has its own, in plain C with % operators).
//
// The map is the Carter-Wegman family stated in roast.h (hash h1 / h2 and sign g of Section 4.1 of
// arXiv 2207.10702).  Every `mod` is a Barrett reduction with a reciprocal prepared once on the
// host, so the device never runs a 64-bit divide.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "roast.h"

namespace roast {

// x mod d for any 64-bit x, using mu = floor(2^64 / d) (all-ones when d == 1).
// floor(x*mu / 2^64) is the true quotient or one less, so one conditional subtract finishes it.
struct Barrett {
  uint64_t d;
  uint64_t mu;
};

inline Barrett make_barrett(uint64_t d) {
  Barrett b;
  b.d = d;
  b.mu = (d <= 1) ? ~0ull : (uint64_t)((((unsigned __int128)1) << 64) / d);
  return b;
}

__host__ __device__ inline uint64_t mulhi64(uint64_t a, uint64_t b) {
#if defined(__HIP_DEVICE_COMPILE__)
  return __umul64hi(a, b);
#else
  return (uint64_t)(((unsigned __int128)a * b) >> 64);
#endif
}

__host__ __device__ inline uint64_t bmod(uint64_t x, const Barrett& b) {
  uint64_t q = mulhi64(x, b.mu);
  uint64_t r = x - q * b.d;
  return r >= b.d ? r - b.d : r;
}

// Everything a kernel needs to place a block; passed by value as a kernel argument.
struct HashDev {
  Barrett P;      // prime modulus
  Barrett slots;  // number of legal offsets / align
  uint64_t a0, a1, a2, a3;
  uint64_t s0, s1, s2, s3;
  uint32_t align;
  uint32_t use_sign;
  uint32_t slots_mu32;  // floor(2^32 / slots) when slots < 2^32 (0 otherwise: then u mod slots == u)
};

// block = scalars per block (Z1*Z2 or Z).  Caller has validated m_size >= block, align >= 1.
inline HashDev make_hash_dev(const roast_hash& h, int64_t m_size, int64_t block) {
  HashDev d;
  d.P = make_barrett(h.P);
  d.slots = make_barrett((uint64_t)(m_size - block) / h.align + 1);
  d.a0 = h.a0; d.a1 = h.a1; d.a2 = h.a2; d.a3 = h.a3;
  d.s0 = h.s0; d.s1 = h.s1; d.s2 = h.s2; d.s3 = h.s3;
  d.align = h.align;
  d.use_sign = h.use_sign;
  d.slots_mu32 = d.slots.d < (1ull << 32) ? (d.slots.d <= 1 ? 0xffffffffu : (uint32_t)((1ull << 32) / d.slots.d)) : 0u;
  return d;
}

// (c0*k0 + c1*k1 + c2*k2 + c3) mod P with keys and products reduced first (no 64-bit overflow
// for any P < 2^32).
__host__ __device__ inline uint64_t cw(const Barrett& P, uint64_t c0, uint64_t c1, uint64_t c2, uint64_t c3,
                                       uint64_t k0, uint64_t k1, uint64_t k2) {
  uint64_t t0 = bmod(c0 * bmod(k0, P), P);
  uint64_t t1 = bmod(c1 * bmod(k1, P), P);
  uint64_t t2 = bmod(c2 * bmod(k2, P), P);
  return bmod(t0 + t1 + t2 + c3, P);
}

__host__ __device__ inline int64_t block_offset(const HashDev& h, uint64_t k0, uint64_t k1, uint64_t k2) {
  uint64_t u = cw(h.P, h.a0, h.a1, h.a2, h.a3, k0, k1, k2);
  return (int64_t)((uint64_t)h.align * bmod(u, h.slots));
}

// +1 or -1: the sign of a block (use_sign == 1) ...
__host__ __device__ inline int block_sign(const HashDev& h, uint64_t k0, uint64_t k1, uint64_t k2) {
  if (h.use_sign != 1) return 1;
  uint64_t v = cw(h.P, h.s0, h.s1, h.s2, h.s3, k0, k1, k2);
  return 1 - 2 * (int)(v & 1ull);
}
// ... or of a single element, keyed by the element's own coordinates (use_sign == 2)
__host__ __device__ inline int elem_sign(const HashDev& h, uint64_t k0, uint64_t k1, uint64_t k2) {
  if (h.use_sign != 2) return 1;
  uint64_t v = cw(h.P, h.s0, h.s1, h.s2, h.s3, k0, k1, k2);
  return 1 - 2 * (int)(v & 1ull);
}

// ---- the same map evaluated incrementally over the last key (used by the lookup kernels, where one
// row has several chunks k2 = 0, 1, 2, ...).  RowHash holds the part that does not depend on k2.
struct RowHash {
  uint32_t u;  // (a0*k0 + a1*k1 + a3) mod P
  uint32_t v;  // (s0*k0 + s1*k1 + s3) mod P
};

__host__ __device__ inline RowHash row_hash(const HashDev& h, uint64_t k0, uint64_t k1) {
  const uint64_t r0 = bmod(k0, h.P), r1 = bmod(k1, h.P);
  RowHash r;
  r.u = (uint32_t)bmod(bmod(h.a0 * r0, h.P) + bmod(h.a1 * r1, h.P) + h.a3, h.P);
  r.v = h.use_sign ? (uint32_t)bmod(bmod(h.s0 * r0, h.P) + bmod(h.s1 * r1, h.P) + h.s3, h.P) : 0u;
  return r;
}

// u mod slots for u < P < 2^32, by a 32-bit Barrett step (or the identity when slots >= 2^32).
__host__ __device__ inline uint32_t mod_slots32(const HashDev& h, uint32_t u) {
  if (h.slots.d >= (1ull << 32)) return u;
  const uint32_t d = (uint32_t)h.slots.d;
#if defined(__HIP_DEVICE_COMPILE__)
  const uint32_t q = __umulhi(u, h.slots_mu32);
#else
  const uint32_t q = (uint32_t)(((uint64_t)u * h.slots_mu32) >> 32);
#endif
  uint32_t r = u - q * d;
  if (r >= d) r -= d;
  if (r >= d) r -= d;      // slots == 1: mu32 saturates and the estimate can be two short
  return r;
}

// Walks k2 = 0, 1, 2, ... for one row: t2 = (a2*k2) mod P and ts = (s2*k2) mod P are advanced by
// one add and one conditional subtract per step.  Valid while k2 < P (the caller checks C <= P).
struct ChunkWalk {
  uint32_t t2, ts;
  __host__ __device__ ChunkWalk() : t2(0u), ts(0u) {}
  __host__ __device__ inline void get(const HashDev& h, const RowHash& r, int64_t* off, int* sgn) const {
    const uint32_t P = (uint32_t)h.P.d;
    uint64_t u = (uint64_t)r.u + t2;
    if (u >= P) u -= P;
    *off = (int64_t)((uint64_t)h.align * mod_slots32(h, (uint32_t)u));
    uint64_t v = (uint64_t)r.v + ts;
    if (v >= P) v -= P;
    *sgn = h.use_sign == 1 ? 1 - 2 * (int)(v & 1ull) : 1;
  }
  __host__ __device__ inline void next(const HashDev& h) {
    const uint32_t P = (uint32_t)h.P.d;
    uint64_t a = (uint64_t)t2 + h.a2;
    if (a >= P) a -= P;
    t2 = (uint32_t)a;
    uint64_t b = (uint64_t)ts + h.s2;
    if (b >= P) b -= P;
    ts = (uint32_t)b;
  }
};

}  // namespace roast
