// Generic ROAST-MM kernels: any H, O, I, any tile size (down to 1x1), fp32 or bf16 activations.
// They are the fp32 path and the fallback for shapes the MFMA kernels do not take.  Plain fp32 FMA
// on a 64x64 output tile per workgroup, both operands staged through LDS; the weight operand is
// read from M element by element through the tile hash (Section 4.1 mapping equation of
// arXiv 2207.10702), with a one-entry per-thread cache of the last tile's offset and sign.
#include "roast_internal.hpp"

namespace roast {
namespace {

constexpr int TB = 64;  // output tile edge
constexpr int TK = 16;  // contraction step

template <typename T> struct Act;
template <> struct Act<float> {
  static constexpr bool kBf16 = false;
  __device__ static float load(const float* p) { return *p; }
  __device__ static void store(float* p, float v) { *p = v; }
};
template <> struct Act<uint16_t> {
  static constexpr bool kBf16 = true;
  __device__ static float load(const uint16_t* p) { return bf16_bits_to_float(*p); }
  __device__ static void store(uint16_t* p, float v) { *p = float_to_bf16_bits(v); }
};

struct TileCache {
  int x = -1, y = -1;
  int64_t off = 0;
  float sgn = 1.f;
};

__device__ inline void tile_of(const MMArgs& a, TileCache& tc, int x, int y) {
  if (x != tc.x || y != tc.y) {
    tc.x = x; tc.y = y;
    tc.off = block_offset(a.hash, a.layer, (uint64_t)x, (uint64_t)y);
    tc.sgn = (float)block_sign(a.hash, a.layer, (uint64_t)x, (uint64_t)y);
  }
}

// sign * M[slot of W[h,o]], rounded to bfloat16 when the activations are bfloat16.
template <bool kBf16>
__device__ inline float w_elem(const MMArgs& a, const float* __restrict__ M, TileCache& tc, int h, int o) {
  const int x = h / a.Z1, y = o / a.Z2;
  tile_of(a, tc, x, y);
  const int64_t pos = (int64_t)a.Z2 * (h - x * a.Z1) + (o - y * a.Z2);
  float v = tc.sgn * M[tc.off + pos];
  if (a.hash.use_sign == 2) v *= (float)elem_sign(a.hash, a.layer, (uint64_t)h, (uint64_t)o);
  if (kBf16) v = bf16_bits_to_float(float_to_bf16_bits(v));
  return v;
}

// C[I x N] = lambda * A[I x K] * B, with B(k,n) = W(k,n) (forward: K=H, N=O) or W(n,k) (dX: K=O, N=H).
template <typename T, bool DX>
__global__ __launch_bounds__(256) void k_generic_mm(MMArgs a, const T* __restrict__ A, int64_t lda,
                                                    const float* __restrict__ M, T* __restrict__ C, int64_t ldc) {
  const int K = DX ? (int)a.O : (int)a.H;
  const int N = DX ? (int)a.H : (int)a.O;
  const int I = (int)a.I;
  __shared__ float As[TK][TB + 4];
  __shared__ float Bs[TK][TB + 4];
  const int t = threadIdx.x, tx = t % 16, ty = t / 16;
  const int m0 = blockIdx.y * TB, n0 = blockIdx.x * TB;
  float acc[4][4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;
  TileCache tc;
  for (int k0 = 0; k0 < K; k0 += TK) {
    {
      const int r = t / 4, kb = (t % 4) * 4, gi = m0 + r;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int gk = k0 + kb + j;
        As[kb + j][r] = (gi < I && gk < K) ? Act<T>::load(A + (int64_t)gi * lda + gk) : 0.f;
      }
    }
    {
      const int kk = t / 16, nb = (t % 16) * 4, gk = k0 + kk;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int gn = n0 + nb + j;
        float v = 0.f;
        if (gk < K && gn < N) v = DX ? w_elem<Act<T>::kBf16>(a, M, tc, gn, gk) : w_elem<Act<T>::kBf16>(a, M, tc, gk, gn);
        Bs[kk][nb + j] = v;
      }
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) av[r] = As[kk][ty * 4 + r];
#pragma unroll
      for (int c = 0; c < 4; ++c) bv[c] = Bs[kk][tx * 4 + c];
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(av[r], bv[c], acc[r][c]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int gi = m0 + ty * 4 + r;
    if (gi >= I) continue;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int gn = n0 + tx * 4 + c;
      if (gn < N) Act<T>::store(C + (int64_t)gi * ldc + gn, a.lambda * acc[r][c]);
    }
  }
}

// G[h,o] = sum_{i in split} X[i,h] * dY[i,o] on a 64x64 tile of (h,o); then either
//   dM[slot(h,o)] += lambda*sign*G   (Gws == nullptr), or
//   Gws[split][h][o] = G             (raw partial products for the deterministic reduction).
template <typename T>
__global__ __launch_bounds__(256) void k_generic_dm(MMArgs a, const T* __restrict__ X, int64_t ldx,
                                                    const T* __restrict__ dY, int64_t ldy, float* __restrict__ dM,
                                                    float* __restrict__ Gws, int rows_per_split) {
  const int H = (int)a.H, O = (int)a.O, I = (int)a.I;
  __shared__ float Xs[TK][TB + 4];
  __shared__ float Ds[TK][TB + 4];
  const int t = threadIdx.x, tx = t % 16, ty = t / 16;
  const int h0 = blockIdx.y * TB, o0 = blockIdx.x * TB;
  const int i_begin = blockIdx.z * rows_per_split;
  const int i_end = min(I, i_begin + rows_per_split);
  float acc[4][4];
#pragma unroll
  for (int r = 0; r < 4; ++r)
#pragma unroll
    for (int c = 0; c < 4; ++c) acc[r][c] = 0.f;
  for (int i0 = i_begin; i0 < i_end; i0 += TK) {
    const int ii = t / 16, cb = (t % 16) * 4, gi = i0 + ii;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int gh = h0 + cb + j, go = o0 + cb + j;
      Xs[ii][cb + j] = (gi < i_end && gh < H) ? Act<T>::load(X + (int64_t)gi * ldx + gh) : 0.f;
      Ds[ii][cb + j] = (gi < i_end && go < O) ? Act<T>::load(dY + (int64_t)gi * ldy + go) : 0.f;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < TK; ++kk) {
      float av[4], bv[4];
#pragma unroll
      for (int r = 0; r < 4; ++r) av[r] = Xs[kk][ty * 4 + r];
#pragma unroll
      for (int c = 0; c < 4; ++c) bv[c] = Ds[kk][tx * 4 + c];
#pragma unroll
      for (int r = 0; r < 4; ++r)
#pragma unroll
        for (int c = 0; c < 4; ++c) acc[r][c] = fmaf(av[r], bv[c], acc[r][c]);
    }
    __syncthreads();
  }
  TileCache tc;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int gh = h0 + ty * 4 + r;
    if (gh >= H) continue;
#pragma unroll
    for (int c = 0; c < 4; ++c) {
      const int go = o0 + tx * 4 + c;
      if (go >= O) continue;
      if (Gws) {
        Gws[((int64_t)blockIdx.z * H + gh) * O + go] = acc[r][c];
      } else {
        const int x = gh / a.Z1, y = go / a.Z2;
        tile_of(a, tc, x, y);
        const int64_t pos = (int64_t)a.Z2 * (gh - x * a.Z1) + (go - y * a.Z2);
        const float es = a.hash.use_sign == 2 ? (float)elem_sign(a.hash, a.layer, (uint64_t)gh, (uint64_t)go) : 1.f;
        unsafeAtomicAdd(dM + tc.off + pos, a.lambda * tc.sgn * es * acc[r][c]);
      }
    }
  }
}

__global__ void k_tile_index(MMArgs a, int64_t* __restrict__ off, int8_t* __restrict__ sgn) {
  const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (t >= a.nTx * a.nTy) return;
  const uint64_t x = (uint64_t)(t / a.nTy), y = (uint64_t)(t % a.nTy);
  off[t] = block_offset(a.hash, a.layer, x, y);
  sgn[t] = (int8_t)block_sign(a.hash, a.layer, x, y);
}

inline dim3 grid2(int64_t cols, int64_t rows) { return dim3((unsigned)((cols + TB - 1) / TB), (unsigned)((rows + TB - 1) / TB), 1); }

}  // namespace

roast_status generic_mm_fwd(const MMArgs& a, roast_dtype dt, const void* X, int64_t ldx, const float* M, void* Y,
                            int64_t ldy, hipStream_t s) {
  const dim3 g = grid2(a.O, a.I);
  if (g.y > 65535) return ROAST_ERR_UNSUPPORTED;
  if (dt == ROAST_F32)
    hipLaunchKernelGGL((k_generic_mm<float, false>), g, dim3(256), 0, s, a, (const float*)X, ldx, M, (float*)Y, ldy);
  else
    hipLaunchKernelGGL((k_generic_mm<uint16_t, false>), g, dim3(256), 0, s, a, (const uint16_t*)X, ldx, M,
                       (uint16_t*)Y, ldy);
  return hip_status(hipGetLastError());
}

roast_status generic_mm_bwd_dx(const MMArgs& a, roast_dtype dt, const void* dY, int64_t ldy, const float* M,
                               void* dX, int64_t ldx, hipStream_t s) {
  const dim3 g = grid2(a.H, a.I);
  if (g.y > 65535) return ROAST_ERR_UNSUPPORTED;
  if (dt == ROAST_F32)
    hipLaunchKernelGGL((k_generic_mm<float, true>), g, dim3(256), 0, s, a, (const float*)dY, ldy, M, (float*)dX, ldx);
  else
    hipLaunchKernelGGL((k_generic_mm<uint16_t, true>), g, dim3(256), 0, s, a, (const uint16_t*)dY, ldy, M,
                       (uint16_t*)dX, ldx);
  return hip_status(hipGetLastError());
}

// Launch the generic dM product with `splits` partitions of the I rows.
roast_status generic_dm_launch(const MMArgs& a, roast_dtype dt, const void* X, int64_t ldx, const void* dY,
                               int64_t ldy, float* dM, float* Gws, int splits, hipStream_t s) {
  dim3 g = grid2(a.O, a.H);
  if (g.y > 65535 || splits < 1 || splits > 65535) return ROAST_ERR_UNSUPPORTED;
  g.z = (unsigned)splits;
  int rows_per_split = (int)((a.I + splits - 1) / splits);
  rows_per_split = (rows_per_split + TK - 1) / TK * TK;
  if (dt == ROAST_F32)
    hipLaunchKernelGGL((k_generic_dm<float>), g, dim3(256), 0, s, a, (const float*)X, ldx, (const float*)dY, ldy,
                       dM, Gws, rows_per_split);
  else
    hipLaunchKernelGGL((k_generic_dm<uint16_t>), g, dim3(256), 0, s, a, (const uint16_t*)X, ldx,
                       (const uint16_t*)dY, ldy, dM, Gws, rows_per_split);
  return hip_status(hipGetLastError());
}

roast_status generic_mm_bwd_dM_atomic(const MMArgs& a, roast_dtype dt, const void* X, int64_t ldx, const void* dY,
                                      int64_t ldy, float* dM, hipStream_t s) {
  const int64_t tiles = ((a.O + TB - 1) / TB) * ((a.H + TB - 1) / TB);
  int64_t splits = (1024 + tiles - 1) / tiles;            // aim for >= 1024 workgroups
  const int64_t max_splits = (a.I + 4 * TK - 1) / (4 * TK);  // at least 64 rows per split
  if (splits > max_splits) splits = max_splits;
  if (splits < 1) splits = 1;
  return generic_dm_launch(a, dt, X, ldx, dY, ldy, dM, nullptr, (int)splits, s);
}

roast_status tile_index_launch(const MMArgs& a, int64_t* off, int8_t* sgn, hipStream_t s) {
  const int64_t n = a.nTx * a.nTy;
  hipLaunchKernelGGL(k_tile_index, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, a, off, sgn);
  return hip_status(hipGetLastError());
}

}  // namespace roast
