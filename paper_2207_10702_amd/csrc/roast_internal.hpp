// Internal declarations shared by the library's translation units (not part of the C-ABI).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "roast.h"
#include "roast_hash.hpp"

namespace roast {

// One validated ROAST-MM call.
struct MMArgs {
  int64_t I, H, O;
  int32_t Z1, Z2;
  int64_t nTx, nTy;  // tile grid
  int64_t m_size;
  uint32_t layer;
  float lambda;
  HashDev hash;
};

// One validated lookup call.
struct EmbedArgs {
  int64_t N, D;
  int32_t Z;
  int64_t C;  // chunks per row = ceil(D/Z)
  int64_t m_size;
  float lambda;
  HashDev hash;
  // pooled (bag-sum) gradient only: lookup n takes its gradient row from dOut[bag of n] instead of
  // dOut[n]; bag b covers lookups [bag_off[b], bag_off[b+1]).  nullptr / 0 for per-lookup calls.
  const int64_t* bag_off;
  int64_t B;
};

inline roast_status hip_status(hipError_t e) { return e == hipSuccess ? ROAST_OK : ROAST_ERR_HIP; }

// bfloat16 <-> float on raw bit patterns (round to nearest even; NaN stays NaN).
__host__ __device__ inline float bf16_bits_to_float(uint16_t b) {
  union { uint32_t u; float f; } v;
  v.u = (uint32_t)b << 16;
  return v.f;
}
__host__ __device__ inline uint16_t float_to_bf16_bits(float f) {
  union { uint32_t u; float f; } v;
  v.f = f;
  if ((v.u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((v.u >> 16) | 0x40u);
  v.u += 0x7fffu + ((v.u >> 16) & 1u);
  return (uint16_t)(v.u >> 16);
}

// ---- generic kernels: any shape, any tile size, fp32 or bf16 activations (roast_mm_generic.hip)
roast_status generic_mm_fwd(const MMArgs& a, roast_dtype dt, const void* X, int64_t ldx, const float* M,
                            void* Y, int64_t ldy, hipStream_t s);
roast_status generic_mm_bwd_dx(const MMArgs& a, roast_dtype dt, const void* dY, int64_t ldy, const float* M,
                               void* dX, int64_t ldx, hipStream_t s);
roast_status generic_mm_bwd_dM_atomic(const MMArgs& a, roast_dtype dt, const void* X, int64_t ldx,
                                      const void* dY, int64_t ldy, float* dM, hipStream_t s);

// Generic dM product with an explicit number of I-splits; Gws as for mfma_mm_bwd_dM below.
roast_status generic_dm_launch(const MMArgs& a, roast_dtype dt, const void* X, int64_t ldx, const void* dY,
                               int64_t ldy, float* dM, float* Gws, int splits, hipStream_t s);

// ---- ATOMIC mode with a workspace: per-split products to ws, then one scatter (roast_reduce.hip)
// Number of parts the contraction (over the I rows) of the dM product is cut into when the output
// has `tiles` workgroup tiles.  The 256 CUs hold one workgroup each, so a launch runs in
// ceil(tiles*s/256) rounds of ceil(steps/s) 64-row steps (1.38 us each, measured) plus about 8 us
// per workgroup; with the atomic epilogue every part also adds all `weights` = H*O products into
// dM, and the chip adds 0.28 M of them per microsecond (weights = 0: no atomic epilogue).  The s
// with the least estimate wins, ties go to fewer parts.  A function of the shape only, so results
// do not depend on the machine's state.
inline int dm_pick_splits(int64_t tiles, int64_t I, int64_t weights) {
  const int64_t steps = (I + 63) / 64;
  int best = 1;
  double best_cost = 1e300;
  for (int s = 1; s <= 16 && (s == 1 || steps / s >= 4); ++s) {
    const double cost = (double)((tiles * s + 255) / 256) * ((double)((steps + s - 1) / s) * 1.38 + 8.0) +
                        (double)s * (double)weights / 0.28e6;
    if (cost < best_cost) { best_cost = cost; best = s; }
  }
  return best;
}
// Parts of the contraction axis (length K) for the forward / dX products when a workspace for fp32
// partial outputs is given: same model, plus about 8 steps for the pass that sums the parts.
inline int mm_pick_splits(int64_t tiles, int64_t K) {
  const int64_t steps = (K + 63) / 64;
  int best = 1;
  int64_t best_cost = INT64_MAX;
  for (int s = 1; s <= 16 && (s == 1 || steps / s >= 4); ++s) {
    const int64_t cost = ((tiles * s + 255) / 256) * ((steps + s - 1) / s + 8) + (s > 1 ? 8 : 0);
    if (cost < best_cost) { best_cost = cost; best = s; }
  }
  return best;
}
size_t dm_ws_workspace_bytes(const MMArgs& a);           // 0: not applicable (direct atomics are used)
roast_status dm_ws_run(const MMArgs& a, const void* X, int64_t ldx, const void* dY, int64_t ldy, float* dM, void* ws,
                       hipStream_t s);

// ---- deterministic dM reduction (roast_reduce.hip)
// Workspace layout: [G: S*H*O floats][tile keys: nT uint64][sorted tile ids: nT uint32]
int dm_det_splits(const MMArgs& a);                       // S: how many partial products of G are kept
size_t dm_det_workspace_bytes(const MMArgs& a);
roast_status dm_det_run(const MMArgs& a, roast_dtype dt, const void* X, int64_t ldx, const void* dY,
                        int64_t ldy, float* dM, void* ws, hipStream_t s);

// ---- bf16 MFMA kernels (roast_mm_mfma.hip): return ROAST_ERR_UNSUPPORTED when the shape does not
// meet their divisibility rules; the caller then falls back to the generic kernels.
// M_bf16 (optional): bf16 copy of M made by shadow_bf16_launch; halves the weight traffic.
int64_t shadow_stride(int64_t m_size);   // elements between the two copies of the bf16 shadow (a multiple of 64)
roast_status shadow_bf16_launch(const float* M, int64_t m_size, void* shadow, hipStream_t s);
// ws (optional): room for mfma_*_splits() fp32 partial outputs [parts][I][columns]; when given and the
// shape has too few output tiles to fill the chip, the contraction axis is split over workgroups.
int mfma_fwd_splits(const MMArgs& a);    // 1: no split (or shape not handled by these kernels)
int mfma_fwd_strip(const MMArgs& a, bool shadow);   // consecutive column blocks per workgroup (1: none) when the contraction is not split
int mfma_dx_strip(const MMArgs& a, bool shadow);
int mfma_dx_splits(const MMArgs& a);
roast_status mfma_mm_fwd(const MMArgs& a, const void* X, int64_t ldx, const float* M, const void* M_bf16, void* Y,
                         int64_t ldy, float* ws, hipStream_t s);
roast_status mfma_mm_bwd_dx(const MMArgs& a, const void* dY, int64_t ldy, const float* M, const void* M_bf16,
                            void* dX, int64_t ldx, float* ws, hipStream_t s);
// fp32 operands on the bf16 matrix cores (three bfloat16 planes per operand, six plane products):
// workspace bytes (0: shape not covered) and the three products; UNSUPPORTED -> generic kernels.
size_t x3_fwd_workspace(const MMArgs& a);
size_t x3_dx_workspace(const MMArgs& a);
size_t x3_dm_workspace(const MMArgs& a);
// M_planes (optional): the three plane shadows of M made by m_planes_launch; NULL = made per call in ws
size_t m_planes_bytes(int64_t m_size);
roast_status m_planes_launch(const float* M, int64_t m_size, void* planes, hipStream_t s);
roast_status x3_mm_fwd(const MMArgs& a, const float* X, int64_t ldx, const float* M, const void* M_planes, float* Y,
                       int64_t ldy, void* ws, hipStream_t s);
roast_status x3_mm_bwd_dx(const MMArgs& a, const float* dY, int64_t ldy, const float* M, const void* M_planes,
                          float* dX, int64_t ldx, void* ws, hipStream_t s);
roast_status x3_mm_bwd_dM(const MMArgs& a, const float* X, int64_t ldx, const float* dY, int64_t ldy, float* dM,
                          void* ws, hipStream_t s);
// Gws == nullptr: atomically add lambda*sign*G into dM.  Gws != nullptr: store raw per-split G there
// ([splits][H][O] floats) for the deterministic reduction; `splits` must equal dm_det_splits().
roast_status mfma_mm_bwd_dM(const MMArgs& a, const void* X, int64_t ldx, const void* dY, int64_t ldy, float* dM,
                            float* Gws, int splits, hipStream_t s);

// ---- lookup kernels (roast_embed.hip)
roast_status embed_fwd_launch(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, const float* M,
                              float* out, hipStream_t s);
// ws may be null (or too small): the gradient then goes straight to dM with global atomics.
// out[b, :] = sum of the rows of the lookups of bag b (a.bag_off, a.B set)
roast_status embed_bag_fwd_launch(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, const float* M,
                                  float* out, hipStream_t s);
size_t embed_bucket_workspace_bytes(const EmbedArgs& a);
roast_status embed_bwd_atomic_launch(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables,
                                     const float* dOut, float* dM, void* ws, size_t ws_bytes, hipStream_t s);
size_t embed_det_workspace_bytes(const EmbedArgs& a);
roast_status embed_bwd_det_run(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, const float* dOut,
                               float* dM, void* ws, hipStream_t s);
// the same gradient with its workspace in a static device array (no caller buffer); WORKSPACE when
// the call needs more than embed_static_scratch_bytes()
size_t embed_static_scratch_bytes();
roast_status embed_bwd_static_run(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, const float* dOut,
                                  float* dM, bool deterministic, hipStream_t s);
roast_status optim_launch(const roast_optim_desc& d, int64_t m_size, float* M, float* dM, float* st1, float* st2,
                          void* shadow, hipStream_t s);
roast_status chunk_index_launch(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, int64_t* off,
                                int8_t* sgn, hipStream_t s);
roast_status tile_index_launch(const MMArgs& a, int64_t* off, int8_t* sgn, hipStream_t s);

}  // namespace roast
