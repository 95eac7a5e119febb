// bf16 MFMA kernels for ROAST-MM on gfx950 (Algorithm 1 and the Section 3.3 gradients of
// arXiv 2207.10702): forward Y = X*W, dX = dY*W^T and the per-tile products of dM = scatter(X^T*dY),
// with W recovered from M tile by tile and never written to memory.
//
// One workgroup = 256 threads = 4 waves (2 x 2) computes a BM x BN block of the output with
// v_mfma_f32_32x32x16_bf16; each wave owns a (BM/2) x (BN/2) sub-block held in fp32 accumulators.
// The contraction runs in steps of BK = 64 through two LDS stages (global -> registers -> LDS while
// the MFMAs of the previous step run).  Operands sit in LDS in one of two layouts:
//   KMAJ: [row][k], 128-byte rows, 16-byte chunks XOR-swizzled by (row & 7); a lane fetches its
//         8 contraction values with one ds_read_b128.  Used when memory is contraction-contiguous
//         (X in forward, dY in dX, and the M tile in dX where the tile's rows run along O).
//   MMAJ: [k][col], rows padded by 64 bytes; a lane fetches its values with two transposing reads
//         (ds_read_b64_tr_b16).  Used when memory is contiguous along the output dimension
//         (the M tile in forward; X and dY in dM, whose contraction runs over the token rows).
// The weight operand is produced on the fly: fp32 values of M at the tile's hashed offset are
// multiplied by the tile's sign, rounded to bf16 and written to LDS.  The tile table (offset, sign)
// of the tiles a workgroup touches is computed by its own threads into LDS at kernel start.
// lambda is applied to the fp32 accumulators in the epilogue.
#include "roast_internal.hpp"

namespace roast {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short short4v __attribute__((ext_vector_type(4)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));

struct __attribute__((packed, aligned(4))) f4u {  // 4 floats, 4-byte aligned (tile bases are arbitrary)
  float v[4];
};

constexpr int BK = 64;
constexpr int kMaxTable = 1024;  // tile-table entries a workgroup may need
enum { MODE_FWD = 0, MODE_DX = 1, MODE_DM = 2 };

__device__ inline uint32_t pack_bf16x2(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 r = {(__bf16)a, (__bf16)b};
  return __builtin_bit_cast(uint32_t, r);
}

// ---- LDS addressing (byte offsets inside one operand tile)
__device__ inline int kmaj_off(int row, int chunk) { return row * 128 + ((chunk ^ (row & 7)) << 4); }
template <int COLS> struct MMaj {
  static constexpr int kStride = COLS * 2 + 64;           // bytes per k-row
  static constexpr int kBytes = BK * kStride;
};
template <int ROWS> struct KMaj { static constexpr int kBytes = ROWS * 128; };

// Fragment of a 32-row block for one k16 sub-step from a KMAJ tile.
__device__ inline bf16x8 frag_kmaj(const char* tile, int row0, int ks, int lane) {
  const int row = row0 + (lane & 31);
  const int chunk = ks * 2 + (lane >> 5);
  return *reinterpret_cast<const bf16x8*>(tile + kmaj_off(row, chunk));
}
// The same fragment from an MMAJ tile via two transposing reads.
template <int STRIDE>
__device__ inline bf16x8 frag_mmaj(const char* tile, int col0, int ks, int lane) {
  const int g = lane >> 4, r = lane & 15, q = r & 3, j = r >> 2;
  const int krow = ks * 16 + 8 * (g >> 1) + j;
  const int col = col0 + 16 * (g & 1) + 4 * q;
  typedef short4v __attribute__((address_space(3))) * lds_p;
  const char* p = tile + krow * STRIDE + col * 2;
  short4v lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p));
  short4v hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_p)(p + 4 * STRIDE));
  typedef short short8v __attribute__((ext_vector_type(8)));
  short8v v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

struct KernArgs {
  MMArgs a;
  const uint16_t* A;   // FWD: X, DX: dY, DM: X
  int64_t lda;
  const uint16_t* B;   // DM: dY
  int64_t ldb;
  const float* M;      // FWD / DX
  uint16_t* C;         // FWD: Y, DX: dX
  int64_t ldc;
  float* dM;           // DM, atomic mode
  float* G;            // DM, deterministic mode: raw products [split][H][O]
  int rows_per_split;  // DM
};

template <int MODE, int BM, int BN>
__global__ __launch_bounds__(256, 1) void k_roast_mfma(KernArgs p) {
  constexpr bool A_KMAJ = (MODE != MODE_DM);
  constexpr bool B_KMAJ = (MODE == MODE_DX);
  constexpr int A_BYTES = A_KMAJ ? KMaj<BM>::kBytes : MMaj<BM>::kBytes;
  constexpr int B_BYTES = B_KMAJ ? KMaj<BN>::kBytes : MMaj<BN>::kBytes;
  constexpr int STAGE = A_BYTES + B_BYTES;
  constexpr int MI = BM / 64, NI = BN / 64;      // 32x32 blocks per wave in each direction
  constexpr int A_STRIDE = MMaj<BM>::kStride, B_STRIDE = MMaj<BN>::kStride;

  extern __shared__ __attribute__((aligned(128))) char smem[];
  int64_t* s_off = reinterpret_cast<int64_t*>(smem + 2 * STAGE);
  float* s_sgn = reinterpret_cast<float*>(smem + 2 * STAGE + kMaxTable * 8);

  const MMArgs& a = p.a;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int I = (int)a.I;
  // output block and contraction range
  const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
  const int Mdim = MODE == MODE_DM ? (int)a.H : I;                      // rows of the output block space
  const int Ndim = MODE == MODE_FWD ? (int)a.O : (MODE == MODE_DX ? (int)a.H : (int)a.O);
  int k_begin = 0, k_end = MODE == MODE_FWD ? (int)a.H : (MODE == MODE_DX ? (int)a.O : I);
  if (MODE == MODE_DM) {
    k_begin = blockIdx.z * p.rows_per_split;
    k_end = min(I, k_begin + p.rows_per_split);
  }
  const int nsteps = (k_end - k_begin + BK - 1) / BK;

  // ---- tile table
  // FWD: entry [kt * TN + yl] for tile (x = kt, y = n0/Z2 + yl), TN = tiles spanned by BN along O
  // DX : entry [kt * TN + xl] for tile (x = n0/Z1 + xl, y = kt), TN = tiles spanned by BN along H
  // DM : entry [xl * TN + yl] for tile (x = m0/Z1 + xl, y = n0/Z2 + yl)
  int TN = 1;
  if (MODE == MODE_FWD) {
    const int y0 = n0 / a.Z2;
    TN = (min(n0 + BN, (int)a.O) - 1) / a.Z2 - y0 + 1;
    const int cnt = (int)a.nTx * TN;
    for (int e = tid; e < cnt; e += 256) {
      const uint64_t x = e / TN, y = y0 + e % TN;
      s_off[e] = block_offset(a.hash, a.layer, x, y);
      s_sgn[e] = (float)block_sign(a.hash, a.layer, x, y);
    }
  } else if (MODE == MODE_DX) {
    const int x0 = n0 / a.Z1;
    TN = (min(n0 + BN, (int)a.H) - 1) / a.Z1 - x0 + 1;
    const int cnt = (int)a.nTy * TN;
    for (int e = tid; e < cnt; e += 256) {
      const uint64_t y = e / TN, x = x0 + e % TN;
      s_off[e] = block_offset(a.hash, a.layer, x, y);
      s_sgn[e] = (float)block_sign(a.hash, a.layer, x, y);
    }
  } else {
    const int x0 = m0 / a.Z1, y0 = n0 / a.Z2;
    const int TM = (min(m0 + BM, (int)a.H) - 1) / a.Z1 - x0 + 1;
    TN = (min(n0 + BN, (int)a.O) - 1) / a.Z2 - y0 + 1;
    for (int e = tid; e < TM * TN; e += 256) {
      const uint64_t x = x0 + e / TN, y = y0 + e % TN;
      s_off[e] = block_offset(a.hash, a.layer, x, y);
      s_sgn[e] = (float)block_sign(a.hash, a.layer, x, y);
    }
  }
  __syncthreads();

  // ---- staging registers
  constexpr int A_LOADS = BM * BK * 2 / 16 / 256;            // 16-byte loads per thread for the A tile
  constexpr int BW_LOADS = BK * BN / 4 / 256;                // float4 loads per thread for a weight tile
  constexpr int BD_LOADS = BK * BN * 2 / 16 / 256;           // 16-byte loads per thread for dY (DM)
  uint4v a_reg[A_LOADS];
  floatx4 bw_reg[MODE == MODE_DM ? 1 : BW_LOADS];
  uint4v bd_reg[MODE == MODE_DM ? BD_LOADS : 1];
  float bw_sgn[MODE == MODE_DX ? BW_LOADS : 1];

  auto load_global = [&](int step) {
    const int k0 = k_begin + step * BK;
    if (A_KMAJ) {
      // A tile: BM rows x 64 k, 8 chunks of 16 bytes per row
      const int c = tid & 7, r0 = tid >> 3;
#pragma unroll
      for (int q = 0; q < A_LOADS; ++q) {
        const int row = r0 + 32 * q;
        uint4v v = {0u, 0u, 0u, 0u};
        if (m0 + row < I) v = *reinterpret_cast<const uint4v*>(p.A + (int64_t)(m0 + row) * p.lda + k0 + 8 * c);
        a_reg[q] = v;
      }
    } else {
      // DM: A tile = X[i][h0 .. h0+BM): BK rows of BM columns, BM/8 chunks per row
      constexpr int CPR = BM / 8, RPP = 256 / CPR;
      const int c = tid % CPR, r0 = tid / CPR;
#pragma unroll
      for (int q = 0; q < A_LOADS; ++q) {
        const int kr = r0 + RPP * q;
        uint4v v = {0u, 0u, 0u, 0u};
        if (k0 + kr < k_end && m0 + 8 * c < (int)a.H)
          v = *reinterpret_cast<const uint4v*>(p.A + (int64_t)(k0 + kr) * p.lda + m0 + 8 * c);
        a_reg[q] = v;
      }
    }
    if (MODE == MODE_FWD) {
      // weight tile [k][n]: BN/4 float4 per k-row
      constexpr int CPR = BN / 4, RPP = 256 / CPR;
      const int c4 = tid % CPR, r0 = tid / CPR;
      const int n = n0 + 4 * c4;
      const int yl = n / a.Z2 - n0 / a.Z2;
      const int e = (k0 / a.Z1) * TN + yl;
      const bool ok = n < (int)a.O;
      const float* base = p.M + (ok ? s_off[e] : 0) + (int64_t)a.Z2 * (k0 % a.Z1) + (n % a.Z2);
      const float sg = ok ? s_sgn[e] : 0.f;
#pragma unroll
      for (int q = 0; q < BW_LOADS; ++q) {
        const int kr = r0 + RPP * q;
        floatx4 v = {0.f, 0.f, 0.f, 0.f};
        if (ok) {
          const f4u m = *reinterpret_cast<const f4u*>(base + (int64_t)kr * a.Z2);
          v = floatx4{m.v[0] * sg, m.v[1] * sg, m.v[2] * sg, m.v[3] * sg};
        }
        bw_reg[q] = v;
      }
    } else if (MODE == MODE_DX) {
      // weight tile as [n = h][k = o]: 16 float4 per row
      const int c4 = tid & 15, r0 = tid >> 4;
      const int kt = k0 / a.Z2;
#pragma unroll
      for (int q = 0; q < BW_LOADS; ++q) {
        const int nr = r0 + 16 * q;
        const int h = n0 + nr;
        floatx4 v = {0.f, 0.f, 0.f, 0.f};
        float sg = 0.f;
        if (h < (int)a.H) {
          const int xl = h / a.Z1 - n0 / a.Z1;
          const int e = kt * TN + xl;
          sg = s_sgn[e];
          const f4u m = *reinterpret_cast<const f4u*>(p.M + s_off[e] + (int64_t)a.Z2 * (h % a.Z1) + (k0 % a.Z2) + 4 * c4);
          v = floatx4{m.v[0], m.v[1], m.v[2], m.v[3]};
        }
        bw_reg[q] = v;
        bw_sgn[q] = sg;
      }
    } else {
      constexpr int CPR = BN / 8, RPP = 256 / CPR;
      const int c = tid % CPR, r0 = tid / CPR;
#pragma unroll
      for (int q = 0; q < BD_LOADS; ++q) {
        const int kr = r0 + RPP * q;
        uint4v v = {0u, 0u, 0u, 0u};
        if (k0 + kr < k_end && n0 + 8 * c < (int)a.O)
          v = *reinterpret_cast<const uint4v*>(p.B + (int64_t)(k0 + kr) * p.ldb + n0 + 8 * c);
        bd_reg[q] = v;
      }
    }
  };

  auto store_lds = [&](int stage) {
    char* At = smem + stage * STAGE;
    char* Bt = At + A_BYTES;
    if (A_KMAJ) {
      const int c = tid & 7, r0 = tid >> 3;
#pragma unroll
      for (int q = 0; q < A_LOADS; ++q) *reinterpret_cast<uint4v*>(At + kmaj_off(r0 + 32 * q, c)) = a_reg[q];
    } else {
      constexpr int CPR = BM / 8, RPP = 256 / CPR;
      const int c = tid % CPR, r0 = tid / CPR;
#pragma unroll
      for (int q = 0; q < A_LOADS; ++q)
        *reinterpret_cast<uint4v*>(At + (r0 + RPP * q) * A_STRIDE + c * 16) = a_reg[q];
    }
    if (MODE == MODE_FWD) {
      constexpr int CPR = BN / 4, RPP = 256 / CPR;
      const int c4 = tid % CPR, r0 = tid / CPR;
#pragma unroll
      for (int q = 0; q < BW_LOADS; ++q) {
        const floatx4 v = bw_reg[q];
        uint2v w = {pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3])};
        *reinterpret_cast<uint2v*>(Bt + (r0 + RPP * q) * B_STRIDE + c4 * 8) = w;
      }
    } else if (MODE == MODE_DX) {
      const int c4 = tid & 15, r0 = tid >> 4;
#pragma unroll
      for (int q = 0; q < BW_LOADS; ++q) {
        const floatx4 v = bw_reg[q];
        const float sg = bw_sgn[q];
        uint2v w = {pack_bf16x2(v[0] * sg, v[1] * sg), pack_bf16x2(v[2] * sg, v[3] * sg)};
        *reinterpret_cast<uint2v*>(Bt + kmaj_off(r0 + 16 * q, c4 >> 1) + 8 * (c4 & 1)) = w;
      }
    } else {
      constexpr int CPR = BN / 8, RPP = 256 / CPR;
      const int c = tid % CPR, r0 = tid / CPR;
#pragma unroll
      for (int q = 0; q < BD_LOADS; ++q)
        *reinterpret_cast<uint4v*>(Bt + (r0 + RPP * q) * B_STRIDE + c * 16) = bd_reg[q];
    }
  };

  floatx16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  auto compute = [&](int stage) {
    const char* At = smem + stage * STAGE;
    const char* Bt = At + A_BYTES;
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      bf16x8 af[MI], bfr[NI];
#pragma unroll
      for (int i = 0; i < MI; ++i) {
        const int r = wm * (BM / 2) + i * 32;
        af[i] = A_KMAJ ? frag_kmaj(At, r, ks, lane) : frag_mmaj<A_STRIDE>(At, r, ks, lane);
      }
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int c = wn * (BN / 2) + j * 32;
        bfr[j] = B_KMAJ ? frag_kmaj(Bt, c, ks, lane) : frag_mmaj<B_STRIDE>(Bt, c, ks, lane);
      }
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
  };

  if (nsteps > 0) {
    load_global(0);
    store_lds(0);
  }
  __syncthreads();
  for (int s = 0; s < nsteps; ++s) {
    const bool more = s + 1 < nsteps;
    if (more) load_global(s + 1);
    compute(s & 1);
    if (more) store_lds((s + 1) & 1);
    __syncthreads();
  }

  // ---- epilogue.  acc[i][j][e]: row = 8*(e/4) + 4*(lane/32) + e%4, col = lane%32 inside the block.
  const int lr = 4 * (lane >> 5), lc = lane & 31;
  if (MODE != MODE_DM) {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int col = n0 + wn * (BN / 2) + j * 32 + lc;
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int row = m0 + wm * (BM / 2) + i * 32 + 8 * (e >> 2) + lr + (e & 3);
          if (row < Mdim && col < Ndim)
            p.C[(int64_t)row * p.ldc + col] = __builtin_bit_cast(uint16_t, (__bf16)(a.lambda * acc[i][j][e]));
        }
      }
  } else {
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int hb = m0 + wm * (BM / 2) + i * 32;      // block origin: inside one hash tile (Z1, Z2 % 32 == 0)
        const int ob = n0 + wn * (BN / 2) + j * 32;
        if (hb >= (int)a.H || ob >= (int)a.O) continue;
        if (p.G) {
          float* g = p.G + ((int64_t)blockIdx.z * a.H + hb) * a.O + ob + lc;
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int r = 8 * (e >> 2) + lr + (e & 3);
            if (hb + r < (int)a.H && ob + lc < (int)a.O) g[(int64_t)r * a.O] = acc[i][j][e];
          }
        } else {
          const int ent = (hb / a.Z1 - m0 / a.Z1) * TN + (ob / a.Z2 - n0 / a.Z2);
          const float sc = a.lambda * s_sgn[ent];
          float* d = p.dM + s_off[ent] + (int64_t)a.Z2 * (hb % a.Z1) + (ob % a.Z2) + lc;
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int r = 8 * (e >> 2) + lr + (e & 3);
            if (hb + r < (int)a.H && ob + lc < (int)a.O) unsafeAtomicAdd(d + (int64_t)r * a.Z2, sc * acc[i][j][e]);
          }
        }
      }
  }
}

template <int MODE, int BM, int BN>
constexpr int smem_bytes() {
  constexpr int A_BYTES = (MODE != MODE_DM) ? KMaj<BM>::kBytes : MMaj<BM>::kBytes;
  constexpr int B_BYTES = (MODE == MODE_DX) ? KMaj<BN>::kBytes : MMaj<BN>::kBytes;
  return 2 * (A_BYTES + B_BYTES) + kMaxTable * 12;
}

template <int MODE, int BM, int BN>
roast_status launch(const KernArgs& p, dim3 grid, hipStream_t s) {
  constexpr int smem = smem_bytes<MODE, BM, BN>();
  static bool configured = false;   // one attribute call per instantiation per process
  if (!configured) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_roast_mfma<MODE, BM, BN>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
      return ROAST_ERR_HIP;
    configured = true;
  }
  hipLaunchKernelGGL((k_roast_mfma<MODE, BM, BN>), grid, dim3(256), smem, s, p);
  return hip_status(hipGetLastError());
}

inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }
inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }

}  // namespace

roast_status mfma_mm_fwd(const MMArgs& a, const void* X, int64_t ldx, const float* M, void* Y, int64_t ldy,
                         hipStream_t s) {
  if (a.Z1 % BK != 0 || a.H % a.Z1 != 0 || a.Z2 % 4 != 0 || a.O % 4 != 0 || ldx % 8 != 0 || !aligned16(X))
    return ROAST_ERR_UNSUPPORTED;
  constexpr int BM = 256, BN = 256;
  if (a.nTx * cdiv(BN, a.Z2) + a.nTx > kMaxTable) return ROAST_ERR_UNSUPPORTED;
  KernArgs p{};
  p.a = a; p.A = (const uint16_t*)X; p.lda = ldx; p.M = M; p.C = (uint16_t*)Y; p.ldc = ldy;
  const dim3 grid((unsigned)cdiv(a.O, BN), (unsigned)cdiv(a.I, BM), 1);
  if (grid.y > 65535) return ROAST_ERR_UNSUPPORTED;
  return launch<MODE_FWD, BM, BN>(p, grid, s);
}

roast_status mfma_mm_bwd_dx(const MMArgs& a, const void* dY, int64_t ldy, const float* M, void* dX, int64_t ldx,
                            hipStream_t s) {
  if (a.Z2 % BK != 0 || a.O % a.Z2 != 0 || ldy % 8 != 0 || !aligned16(dY)) return ROAST_ERR_UNSUPPORTED;
  constexpr int BM = 256, BN = 256;
  if (a.nTy * cdiv(BN, a.Z1) + a.nTy > kMaxTable) return ROAST_ERR_UNSUPPORTED;
  KernArgs p{};
  p.a = a; p.A = (const uint16_t*)dY; p.lda = ldy; p.M = M; p.C = (uint16_t*)dX; p.ldc = ldx;
  const dim3 grid((unsigned)cdiv(a.H, BN), (unsigned)cdiv(a.I, BM), 1);
  if (grid.y > 65535) return ROAST_ERR_UNSUPPORTED;
  return launch<MODE_DX, BM, BN>(p, grid, s);
}

roast_status mfma_mm_bwd_dM(const MMArgs& a, const void* X, int64_t ldx, const void* dY, int64_t ldy, float* dM,
                            float* Gws, int splits, hipStream_t s) {
  if (a.Z1 % 32 != 0 || a.Z2 % 32 != 0 || a.H % 8 != 0 || a.O % 8 != 0 || ldx % 8 != 0 || ldy % 8 != 0 ||
      !aligned16(X) || !aligned16(dY))
    return ROAST_ERR_UNSUPPORTED;
  constexpr int BM = 256, BN = 256;
  if (cdiv(BM, a.Z1) * cdiv(BN, a.Z2) + cdiv(BM, a.Z1) + cdiv(BN, a.Z2) + 1 > kMaxTable) return ROAST_ERR_UNSUPPORTED;
  const int64_t tiles = cdiv(a.H, BM) * cdiv(a.O, BN);
  if (Gws == nullptr) {
    // enough workgroups to fill 256 CUs a few times over, but at least 4 contraction steps each
    int64_t want = cdiv(768, tiles);
    const int64_t cap = cdiv(a.I, 4 * BK);
    if (want > cap) want = cap;
    if (want < 1) want = 1;
    splits = (int)want;
  }
  if (splits < 1 || splits > 65535) return ROAST_ERR_UNSUPPORTED;
  int64_t rows = cdiv(a.I, splits);
  rows = cdiv(rows, BK) * BK;
  KernArgs p{};
  p.a = a; p.A = (const uint16_t*)X; p.lda = ldx; p.B = (const uint16_t*)dY; p.ldb = ldy; p.dM = dM; p.G = Gws;
  p.rows_per_split = (int)rows;
  const dim3 grid((unsigned)cdiv(a.O, BN), (unsigned)cdiv(a.H, BM), (unsigned)splits);
  if (grid.y > 65535) return ROAST_ERR_UNSUPPORTED;
  return launch<MODE_DM, BM, BN>(p, grid, s);
}

}  // namespace roast
