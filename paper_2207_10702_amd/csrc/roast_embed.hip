// ROAST lookup kernels: out[n, c*Z + o] = lambda * sign * M[offset(table, row, c) + o]
// (lookup equation of Section 3.1 of arXiv 2207.10702) and its scatter-add gradient (Section 3.3).
//
// HBM-bound streaming kernels.  Work item = one chunk of one lookup, numbered g = n*C + c, so that
// consecutive items are consecutive in `out`.  A wave takes 64 consecutive items: each lane hashes
// one item (offset + sign), then the wave walks the 64 items a few at a time, each item served by
// LPI neighbouring lanes that move VEC floats each, with the item's offset and sign fetched from
// the owning lane by a cross-lane shuffle.  With Z = 32 and VEC = 4, eight lanes serve a chunk and
// one step moves 1 KiB of contiguous output.
#include "roast_internal.hpp"

namespace roast {
namespace {

// 4 floats that are only 4-byte aligned in memory (chunk bases are arbitrary offsets into M).
struct __attribute__((packed, aligned(4))) f4u {
  float v[4];
};
typedef float vfloat4 __attribute__((ext_vector_type(4)));

__device__ inline int64_t shfl64(int64_t v, int src) {
  int lo = __shfl((int)(uint32_t)(uint64_t)v, src, 64);
  int hi = __shfl((int)(uint32_t)((uint64_t)v >> 32), src, 64);
  return (int64_t)(((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo);
}

// VEC = 4 requires Z % 4 == 0 and D % Z == 0 (then every chunk is full and out is 16-byte aligned
// per lane, given a 16-byte aligned `out` base).  LPI = lanes per item (power of two <= 64).
template <int VEC, bool BWD>
__global__ __launch_bounds__(256) void k_embed(EmbedArgs a, int lpi_log2, const int64_t* __restrict__ rows,
                                               const uint32_t* __restrict__ tables, const float* __restrict__ M,
                                               float* __restrict__ out, const float* __restrict__ dOut,
                                               float* __restrict__ dM) {
  const int lane = threadIdx.x & 63;
  const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
  const int64_t n_items = a.N * a.C;
  const int64_t g0 = wave * 64;
  if (g0 >= n_items) return;

  // one item per lane: hash it
  int64_t my_off = 0;
  float my_scale = 0.f;
  {
    const int64_t g = g0 + lane;
    if (g < n_items) {
      const int64_t n = g / a.C, c = g - n * a.C;
      const uint64_t r = (uint64_t)rows[n], t = tables[n];
      my_off = block_offset(a.hash, t, r, (uint64_t)c);
      my_scale = a.lambda * (float)block_sign(a.hash, t, r, (uint64_t)c);
    }
  }

  const int lpi = 1 << lpi_log2;
  const int items_per_step = 64 >> lpi_log2;
  const int sub = lane & (lpi - 1);   // my position among the lanes serving one item
  const int which = lane >> lpi_log2; // which item of the step I serve
  const int n_here = (int)min((int64_t)64, n_items - g0);
  for (int j0 = 0; j0 < n_here; j0 += items_per_step) {
    const int j = j0 + which;                     // item inside this wave's batch
    const int src = j < 64 ? j : 63;
    const int64_t off = shfl64(my_off, src);
    const float scale = __shfl(my_scale, src, 64);
    if (j >= n_here) continue;
    const int64_t g = g0 + j;
    const int64_t n = g / a.C, c = g - n * a.C;
    const int len = (int)min((int64_t)a.Z, a.D - c * a.Z);   // last chunk of a row may be short
    const int64_t obase = n * a.D + c * a.Z;
    for (int o = sub * VEC; o < len; o += lpi * VEC) {
      if (VEC == 4) {
        if (!BWD) {
          const f4u m = *reinterpret_cast<const f4u*>(M + off + o);
          vfloat4 v = {scale * m.v[0], scale * m.v[1], scale * m.v[2], scale * m.v[3]};
          __builtin_nontemporal_store(v, reinterpret_cast<vfloat4*>(out + obase + o));
        } else {
          const vfloat4 d = __builtin_nontemporal_load(reinterpret_cast<const vfloat4*>(dOut + obase + o));
          float* p = dM + off + o;
          unsafeAtomicAdd(p + 0, scale * d.x);
          unsafeAtomicAdd(p + 1, scale * d.y);
          unsafeAtomicAdd(p + 2, scale * d.z);
          unsafeAtomicAdd(p + 3, scale * d.w);
        }
      } else {
        if (!BWD) {
          __builtin_nontemporal_store(scale * M[off + o], out + obase + o);
        } else {
          unsafeAtomicAdd(dM + off + o, scale * __builtin_nontemporal_load(dOut + obase + o));
        }
      }
    }
  }
}

__global__ __launch_bounds__(256) void k_chunk_index(EmbedArgs a, const int64_t* __restrict__ rows,
                                                     const uint32_t* __restrict__ tables, int64_t* __restrict__ off,
                                                     int8_t* __restrict__ sgn) {
  const int64_t g = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (g >= a.N * a.C) return;
  const int64_t n = g / a.C, c = g - n * a.C;
  off[g] = block_offset(a.hash, tables[n], (uint64_t)rows[n], (uint64_t)c);
  sgn[g] = (int8_t)block_sign(a.hash, tables[n], (uint64_t)rows[n], (uint64_t)c);
}

template <bool BWD>
roast_status launch_embed(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, const float* M,
                          float* out, const float* dOut, float* dM, hipStream_t s) {
  const int64_t n_items = a.N * a.C;
  const int64_t waves = (n_items + 63) / 64;
  const int64_t blocks = (waves + 3) / 4;
  if (blocks > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
  const void* io = BWD ? (const void*)dOut : (const void*)out;
  const bool vec4 = (a.Z % 4 == 0) && (a.D % a.Z == 0) && (((uintptr_t)io & 15) == 0);
  const int per_lane = vec4 ? 4 : 1;
  int lpi_log2 = 0;
  while ((1 << lpi_log2) < 64 && (int64_t)(1 << lpi_log2) * per_lane < a.Z) ++lpi_log2;
  const dim3 g((unsigned)blocks), b(256);
  if (vec4)
    hipLaunchKernelGGL((k_embed<4, BWD>), g, b, 0, s, a, lpi_log2, rows, tables, M, out, dOut, dM);
  else
    hipLaunchKernelGGL((k_embed<1, BWD>), g, b, 0, s, a, lpi_log2, rows, tables, M, out, dOut, dM);
  return hip_status(hipGetLastError());
}

}  // namespace

roast_status embed_fwd_launch(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, const float* M,
                              float* out, hipStream_t s) {
  return launch_embed<false>(a, rows, tables, M, out, nullptr, nullptr, s);
}

roast_status embed_bwd_atomic_launch(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables,
                                     const float* dOut, float* dM, hipStream_t s) {
  return launch_embed<true>(a, rows, tables, nullptr, nullptr, dOut, dM, s);
}

size_t embed_det_workspace_bytes(const EmbedArgs&) { return 0; }

roast_status embed_bwd_det_run(const EmbedArgs&, const int64_t*, const uint32_t*, const float*, float*, void*,
                               hipStream_t) {
  return ROAST_ERR_UNSUPPORTED;
}

roast_status chunk_index_launch(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, int64_t* off,
                                int8_t* sgn, hipStream_t s) {
  const int64_t n = a.N * a.C;
  const int64_t blocks = (n + 255) / 256;
  if (blocks > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(k_chunk_index, dim3((unsigned)blocks), dim3(256), 0, s, a, rows, tables, off, sgn);
  return hip_status(hipGetLastError());
}

}  // namespace roast
