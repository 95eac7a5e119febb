// ROAST lookup kernels: out[n, c*Z + o] = lambda * sign * M[offset(table, row, c) + o]
// (lookup equation of Section 4.1 of arXiv 2207.10702) and its scatter-add gradient (Section 4.3).
//
// HBM-bound streaming kernels.  Work item = one chunk of one lookup, numbered g = n*C + c, so that
// consecutive items are consecutive in `out`.  The integer work is done per lookup, not per chunk:
// the part of the hash that depends on (table, row) is computed once and the chunk index is walked
// incrementally.  With Z = 32 and VEC = 4, eight lanes serve a chunk and one step of a wave moves
// 1 KiB of contiguous output.
#include <stdlib.h>

#include <algorithm>
#include <atomic>
#include <type_traits>

#include "roast_internal.hpp"

namespace roast {
namespace {

// 4 floats that are only 4-byte aligned in memory (chunk bases are arbitrary offsets into M).
struct __attribute__((packed, aligned(4))) f4u {
  float v[4];
};
typedef float vfloat4 __attribute__((ext_vector_type(4)));

// All chunk keys of one lookup: the row part of the hash once, then one cheap step per chunk.
// `walk` says whether the incremental walk is valid (chunks per row <= P); otherwise every chunk is
// hashed from scratch.  f(c, offset, sign) is called for c = 0 .. C-1.
template <typename F>
__device__ inline void for_each_chunk(const EmbedArgs& a, bool walk, uint64_t table, uint64_t row, F&& f) {
  if (walk) {
    const RowHash rh = row_hash(a.hash, table, row);
    ChunkWalk w;
    for (int64_t c = 0; c < a.C; ++c) {
      int64_t off; int sgn;
      w.get(a.hash, rh, &off, &sgn);
      f(c, off, sgn);
      w.next(a.hash);
    }
  } else {
    for (int64_t c = 0; c < a.C; ++c)
      f(c, block_offset(a.hash, table, row, (uint64_t)c), block_sign(a.hash, table, row, (uint64_t)c));
  }
}

// Pooled gradient: the bag of lookup n = the last b with bag_off[b] <= n (bag_off[0] == 0, so one
// exists; empty bags share their offset with the next one and are skipped by "last").  The result is
// clamped to [0, B-1] whatever the offsets hold, so a malformed offsets array cannot push a read out
// of dOut.
__device__ inline int64_t bag_of(const int64_t* __restrict__ bag_off, int64_t B, int64_t n) {
  int64_t lo = 0, hi = B;
  while (hi - lo > 1) {
    const int64_t mid = (lo + hi) >> 1;
    if (bag_off[mid] <= n) lo = mid; else hi = mid;
  }
  return lo;
}
// row of dOut that lookup n takes its gradient from
__device__ inline int64_t grad_row(const EmbedArgs& a, int64_t n) { return a.bag_off ? bag_of(a.bag_off, a.B, n) : n; }

// Streaming lookup / direct-atomic gradient.  A wave takes 64 lookups: each lane hashes the chunks
// of one lookup into the wave's LDS key list (offset | sign bit, 32-bit), then the wave walks the
// 64*C chunks in order, LPI lanes per chunk, VEC floats per lane.
// VEC = 4 requires Z % 4 == 0 and D % Z == 0 (then every chunk is full and out is 16-byte aligned
// per lane, given a 16-byte aligned base).  Needs |M| < 2^31 and C <= kMaxC.
constexpr int kMaxC = 16;

// slices > 1 (forward only; 2, 4 or 8): M is larger than one XCD's L2, so the gathered reads would
// keep missing it.  The workgroups of XCD group s (workgroups go to the 8 XCDs round-robin) then only
// serve the chunks whose offset lies in the s-th slice of M: every block of 256 lookups is hashed by
// `slices` workgroups on different XCDs (hashing is cheap), each of which gathers from a part of M
// that stays in its L2 and writes its share of the output chunks.
template <int VEC, bool BWD>
__global__ __launch_bounds__(256) void k_embed(EmbedArgs a, int lpi_log2, int walk, const int64_t* __restrict__ rows,
                                               const uint32_t* __restrict__ tables, const float* __restrict__ M,
                                               float* __restrict__ out, const float* __restrict__ dOut,
                                               float* __restrict__ dM, int slices) {
  extern __shared__ uint32_t s_keys[];           // [4 waves][64 * C] keys, then [4 waves][64 * C] selected chunk numbers (16 bit)
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6;
  const int C = (int)a.C;
  uint32_t* keys = s_keys + wv * 64 * C;
  uint16_t* sel = reinterpret_cast<uint16_t*>(s_keys + 4 * 64 * C) + wv * 64 * C;
  const int per = 8 / slices;                    // consecutive lookup blocks per group of 8 workgroups
  const int slice = (int)(blockIdx.x & 7) / per;
  const int64_t lblock = slices == 1 ? (int64_t)blockIdx.x : (int64_t)(blockIdx.x >> 3) * per + (blockIdx.x & (per - 1));
  const int64_t wave = lblock * 4 + wv;
  const int64_t n0 = wave * 64;
  if (n0 >= a.N) return;
  const int rows_here = (int)min((int64_t)64, a.N - n0);
  if (lane < rows_here) {
    const int64_t n = n0 + lane;
    for_each_chunk(a, walk != 0, tables[n], (uint64_t)rows[n], [&](int64_t c, int64_t off, int sgn) {
      keys[lane * C + c] = (uint32_t)off | (sgn < 0 ? 0x80000000u : 0u);
    });
  }
  // the wave reads back what its own lanes wrote: LDS operations of one wave complete in order
  const int lpi = 1 << lpi_log2;
  const int items_per_step = 64 >> lpi_log2;
  const int sub = lane & (lpi - 1);   // my position among the lanes serving one chunk
  const int which = lane >> lpi_log2; // which chunk of the step I serve
  int n_here = rows_here * C;
  const int64_t g0 = n0 * C;
  if (!BWD && slices > 1) {
    // order-preserving selection of this slice's chunks (wave-level: ballot + prefix count)
    const uint32_t lo = (uint32_t)(((int64_t)slice * a.m_size) / slices);
    const uint32_t hi = (uint32_t)(((int64_t)(slice + 1) * a.m_size) / slices);
    int base = 0;
    for (int j0 = 0; j0 < n_here; j0 += 64) {
      const int j = j0 + lane;
      const uint32_t off = j < n_here ? (keys[j] & 0x7fffffffu) : 0xffffffffu;
      const bool mine = j < n_here && off >= lo && off < hi;
      const unsigned long long mask = __ballot(mine);
      if (mine) sel[base + __popcll(mask & ((1ull << lane) - 1ull))] = (uint16_t)j;
      base += __popcll(mask);
    }
    n_here = base;
    if (n_here == 0) return;
  }
  auto chunk_at = [&](int idx) { return (!BWD && slices > 1) ? (int)sel[idx] : idx; };
  if constexpr (VEC == 4 && !BWD) {
    // Forward, full chunks: the gathered reads of M are latency-bound (L2 / memory-side cache), so
    // each wave keeps U chunks per lane group in flight before it stores any of them.
    constexpr int U = 4;
    if (lpi * 4 == a.Z) {          // one 16-byte piece per lane and chunk (Z <= 256): the common case
      for (int j0 = 0; j0 < n_here; j0 += U * items_per_step) {
        vfloat4 v[U];
        int64_t ob[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int j = chunk_at(min(j0 + u * items_per_step + which, n_here - 1));
          const uint32_t key = keys[j];
          const float scale = (key & 0x80000000u) ? -a.lambda : a.lambda;
          const f4u m = *reinterpret_cast<const f4u*>(M + (key & 0x7fffffffu) + sub * 4);
          v[u] = vfloat4{scale * m.v[0], scale * m.v[1], scale * m.v[2], scale * m.v[3]};
          ob[u] = (g0 + j) * a.Z + sub * 4;      // D % Z == 0: chunk g starts at g*Z in the dense output
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (j0 + u * items_per_step + which < n_here) __builtin_nontemporal_store(v[u], reinterpret_cast<vfloat4*>(out + ob[u]));
      }
      return;
    }
  }
  for (int j0 = 0; j0 < n_here; j0 += items_per_step) {
    if (j0 + which >= n_here) continue;
    const int j = chunk_at(j0 + which);
    const uint32_t key = keys[j];
    const int64_t off = key & 0x7fffffffu;
    const float scale = (key & 0x80000000u) ? -a.lambda : a.lambda;
    const int64_t g = g0 + j;
    const int64_t n = g / C, c = g - n * C;
    const int len = (int)min((int64_t)a.Z, a.D - c * a.Z);   // last chunk of a row may be short
    const int64_t obase = (BWD ? grad_row(a, n) : n) * a.D + c * a.Z;
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

// Fallback for huge M (offsets beyond 31 bits) or very many chunks per row: one thread per element.
template <bool BWD>
__global__ __launch_bounds__(256) void k_embed_elem(EmbedArgs a, const int64_t* __restrict__ rows,
                                                    const uint32_t* __restrict__ tables, const float* __restrict__ M,
                                                    float* __restrict__ out, const float* __restrict__ dOut,
                                                    float* __restrict__ dM) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= a.N * a.D) return;
  const int64_t n = e / a.D, i = e - n * a.D, c = i / a.Z, o = i - c * a.Z;
  const int64_t off = block_offset(a.hash, tables[n], (uint64_t)rows[n], (uint64_t)c);
  const float scale = a.lambda * (float)(block_sign(a.hash, tables[n], (uint64_t)rows[n], (uint64_t)c) *
                                         elem_sign(a.hash, tables[n], (uint64_t)rows[n], (uint64_t)i));
  if (!BWD) out[e] = scale * M[off + o];
  else unsafeAtomicAdd(dM + off + o, scale * dOut[grad_row(a, n) * a.D + i]);
}

__global__ __launch_bounds__(256) void k_chunk_index(EmbedArgs a, int walk, const int64_t* __restrict__ rows,
                                                     const uint32_t* __restrict__ tables, int64_t* __restrict__ off,
                                                     int8_t* __restrict__ sgn) {
  const int64_t n = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (n >= a.N) return;
  for_each_chunk(a, walk != 0, tables[n], (uint64_t)rows[n], [&](int64_t c, int64_t o, int s) {
    off[n * a.C + c] = o;
    sgn[n * a.C + c] = (int8_t)s;
  });
}

// Pooled forward: out[b, :] = lambda * sum over the lookups n of bag b of sign_n * M[offset_n(c) + o].
// A workgroup owns `bags_wg` consecutive bags, i.e. one contiguous range of lookups.  It works in
// windows of at most `win` lookups: every lookup of the window is hashed once (one thread per
// lookup, all its chunks, keys to LDS), then each thread walks the part of its bag that lies in the
// window and adds its piece (VEC floats of one chunk) of every row -- gathered reads of M, served by
// L2.  Sums run in lookup order, in fp64, so the result does not depend on the launch shape.
// VEC = 4 requires Z % 4 == 0 and D % 4 == 0 (a piece never straddles a chunk or the row end).
template <int VEC>
__global__ __launch_bounds__(256) void k_embed_bag_fwd(EmbedArgs a, int walk, int tpb, int bags_wg, int win,
                                                       const int64_t* __restrict__ rows,
                                                       const uint32_t* __restrict__ tables,
                                                       const float* __restrict__ M, float* __restrict__ out) {
  extern __shared__ uint32_t s_bag_keys[];       // [win * C]
  const int C = (int)a.C;
  const int64_t b0 = (int64_t)blockIdx.x * bags_wg;
  const int64_t b1 = min(a.B, b0 + bags_wg);
  auto clampN = [&](int64_t v) { return min(max(v, (int64_t)0), a.N); };
  const int64_t n_begin = clampN(a.bag_off[b0]);
  const int64_t n_end = max(n_begin, clampN(a.bag_off[b1]));
  const int bl = threadIdx.x / tpb, tl = threadIdx.x % tpb;
  const int64_t b = b0 + bl;
  const bool active = bl < bags_wg && b < b1;
  int64_t my_begin = 0, my_end = 0;
  if (active) {
    my_begin = min(max(clampN(a.bag_off[b]), n_begin), n_end);
    my_end = min(max(clampN(a.bag_off[b + 1]), my_begin), n_end);
  }
  const int pieces = (int)((a.D + VEC - 1) / VEC);
  for (int p0 = 0; p0 < pieces; p0 += tpb) {           // one pass unless a row has more pieces than tpb
    const int piece = p0 + tl;
    const bool live = active && piece < pieces;
    const int c = live ? (piece * VEC) / a.Z : 0, o = live ? (piece * VEC) % a.Z : 0;
    double acc[VEC];   // a bag may hold thousands of rows: fp64 sums keep the result within one fp32 rounding
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0.0;
    for (int64_t w0 = n_begin; w0 < n_end; w0 += win) {   // uniform trip count for the workgroup
      const int64_t w1 = min(n_end, w0 + win);
      __syncthreads();                                    // the previous window's keys are no longer needed
      for (int64_t n = w0 + threadIdx.x; n < w1; n += 256)
        for_each_chunk(a, walk != 0, tables[n], (uint64_t)rows[n], [&](int64_t cc, int64_t off, int sgn) {
          s_bag_keys[(n - w0) * C + cc] = (uint32_t)off | (sgn < 0 ? 0x80000000u : 0u);
        });
      __syncthreads();
      if (!live) continue;
      const int64_t lo = max(my_begin, w0), hi = min(my_end, w1);
      constexpr int U = 4;
      for (int64_t n = lo; n < hi; n += U) {
        float m[U][VEC];
        float sg[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
          const int64_t nn = min(n + u, hi - 1);
          const uint32_t key = s_bag_keys[(nn - w0) * C + c];
          sg[u] = (n + u < hi) ? ((key & 0x80000000u) ? -1.f : 1.f) : 0.f;
          const float* src = M + (key & 0x7fffffffu) + o;
          if constexpr (VEC == 4) {
            const f4u t = *reinterpret_cast<const f4u*>(src);   // 4-byte aligned: chunk bases are arbitrary
#pragma unroll
            for (int v = 0; v < 4; ++v) m[u][v] = t.v[v];
          } else {
            m[u][0] = src[0];
          }
        }
#pragma unroll
        for (int u = 0; u < U; ++u)
#pragma unroll
          for (int v = 0; v < VEC; ++v) acc[v] += (double)(sg[u] * m[u][v]);
      }
    }
    if (live) {
      float* dst = out + b * a.D + (int64_t)piece * VEC;
      if constexpr (VEC == 4) {
        const double l = (double)a.lambda;
        const vfloat4 r = {(float)(l * acc[0]), (float)(l * acc[1]), (float)(l * acc[2]), (float)(l * acc[3])};
        *reinterpret_cast<vfloat4*>(dst) = r;
      } else {
        dst[0] = (float)((double)a.lambda * acc[0]);
      }
    }
  }
}

// Fallback for huge M or very many chunks per row: one thread per output element.
__global__ __launch_bounds__(256) void k_embed_bag_fwd_elem(EmbedArgs a, const int64_t* __restrict__ rows,
                                                            const uint32_t* __restrict__ tables,
                                                            const float* __restrict__ M, float* __restrict__ out) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= a.B * a.D) return;
  const int64_t b = e / a.D, i = e - b * a.D, c = i / a.Z, o = i - c * a.Z;
  const int64_t n0 = min(max(a.bag_off[b], (int64_t)0), a.N), n1 = min(max(a.bag_off[b + 1], n0), a.N);
  double acc = 0.0;
  for (int64_t n = n0; n < n1; ++n) {
    const int64_t off = block_offset(a.hash, tables[n], (uint64_t)rows[n], (uint64_t)c);
    acc += (double)((float)(block_sign(a.hash, tables[n], (uint64_t)rows[n], (uint64_t)c) *
                            elem_sign(a.hash, tables[n], (uint64_t)rows[n], (uint64_t)i)) * M[off + o]);
  }
  out[e] = (float)((double)a.lambda * acc);
}

inline int walk_ok(const EmbedArgs& a) { return (uint64_t)a.C <= a.hash.P.d ? 1 : 0; }

template <bool BWD>
roast_status launch_embed(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, const float* M,
                          float* out, const float* dOut, float* dM, hipStream_t s) {
  // (the chunk kernels carry one sign per chunk: per-element signs take the per-element kernel)
  if (a.m_size >= (1ll << 31) || a.C > kMaxC || a.hash.use_sign == 2) {
    const int64_t blocks = (a.N * a.D + 255) / 256;
    if (blocks > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
    hipLaunchKernelGGL((k_embed_elem<BWD>), dim3((unsigned)blocks), dim3(256), 0, s, a, rows, tables, M, out, dOut, dM);
    return hip_status(hipGetLastError());
  }
  const int64_t waves = (a.N + 63) / 64;
  int64_t blocks = (waves + 3) / 4;
  const void* io = BWD ? (const void*)dOut : (const void*)out;
  const bool vec4 = (a.Z % 4 == 0) && (a.D % a.Z == 0) && (((uintptr_t)io & 15) == 0);
  const int per_lane = vec4 ? 4 : 1;
  int lpi_log2 = 0;
  while ((1 << lpi_log2) < 64 && (int64_t)(1 << lpi_log2) * per_lane < a.Z) ++lpi_log2;
  // forward over an M that does not fit one XCD's L2 (4 MiB): four slices (measured on a 5 MiB M:
  // 171 us unsliced, 158 / 144 / 189 us with 2 / 4 / 8 slices -- every slice hashes all lookups),
  // eight once a quarter is too large; not for small calls, nor once even an eighth does not fit
  int slices = 1;
  if (!BWD && vec4 && a.N * a.C >= 65536) {
    const int64_t bytes = a.m_size * 4, fit = 3584 * 1024;
    slices = bytes <= fit ? 1 : bytes <= 4 * fit ? 4 : bytes <= 8 * fit ? 8 : 1;
  }
  if (slices > 1) blocks = (blocks + 8 / slices - 1) / (8 / slices) * 8;
  if (blocks > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
  const dim3 g((unsigned)blocks), b(256);
  const size_t lds = (size_t)4 * 64 * a.C * (sizeof(uint32_t) + sizeof(uint16_t));
  if (vec4)
    hipLaunchKernelGGL((k_embed<4, BWD>), g, b, lds, s, a, lpi_log2, walk_ok(a), rows, tables, M, out, dOut, dM, slices);
  else
    hipLaunchKernelGGL((k_embed<1, BWD>), g, b, lds, s, a, lpi_log2, walk_ok(a), rows, tables, M, out, dOut, dM, slices);
  return hip_status(hipGetLastError());
}

// ---------------------------------------------------------------------------------------------
// Bucketed gradient: fp32 global atomics top out near 0.3 T adds/s on this chip, an order of
// magnitude short of what streaming dOut needs, so the scatter-add is reorganised by destination.
//   1. route:  every lookup is hashed once; each of its chunks is appended to the list of the bucket
//              (R consecutive slots of M) its offset falls in.  A workgroup ranks its chunks inside
//              each bucket with LDS counters, reserves list space with one global add per bucket,
//              and writes every entry to reserved base + rank.  Lists have a fixed capacity; a chunk that does not fit
//              is added straight into dM with global atomics instead (rare: only under extreme skew).
//   2. accum:  one workgroup per (bucket, list segment) zeroes an fp64 LDS image of its R (+Z)
//              slots, adds its chunks of dOut into it with LDS atomics, and flushes the image to dM
//              with global atomics -- R adds per workgroup instead of Z adds per chunk.
// Needs Z % 4 == 0, D % Z == 0, C <= kMaxC, |M| < 2^31 and at most kMaxBuckets buckets of at most
// kMaxR slots; other shapes use the direct atomic kernel above.
constexpr int kSeg = 8192;          // chunks per accumulate workgroup
constexpr int kMaxBuckets = 2048;
constexpr int kMaxR = 8192;         // largest bucket (slots); its fp64 LDS image is (kMaxR + Z) * 8 bytes, up to 72 KiB
constexpr int kRouteItems = 8192;   // chunks per route workgroup (lookups per workgroup = kRouteItems / C)
constexpr int kRouteThreads = 512;

struct BucketPlan {
  bool ok;
  int r_log2;          // bucket = offset >> r_log2
  int nb;              // number of buckets
  uint32_t cap;        // list capacity per bucket (entries)
  int64_t n_items;
  size_t cursor_off, list_off, total;
};

inline BucketPlan bucket_plan(const EmbedArgs& a) {
  BucketPlan p{};
  p.n_items = a.N * a.C;
  p.ok = (a.Z % 4 == 0) && (a.D % a.Z == 0) && a.m_size < (1ll << 31) && p.n_items < (1ll << 31) && a.Z <= 1024 &&
         a.C <= kMaxC && a.B * a.C < (1ll << 31) &&  // (B = 0 unless pooled)
         a.hash.use_sign != 2;                       // list entries carry one sign per chunk
  if (!p.ok) return p;
  int r = 12;
  while ((1 << r) < kMaxR && ((a.m_size + (1ll << r) - 1) >> r) > kMaxBuckets) ++r;
  p.r_log2 = r;
  p.nb = (int)((a.m_size + (1ll << r) - 1) >> r);
  if (p.nb > kMaxBuckets) { p.ok = false; return p; }
  // twice the mean load plus one segment: uniform hashing stays far below, skewed ids mostly too
  p.cap = (uint32_t)(2 * (p.n_items / p.nb) + kSeg);
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  size_t o = 0;
  p.cursor_off = o; o += up((size_t)p.nb * 4);
  p.list_off = o;   o += up((size_t)p.nb * p.cap * 8);
  p.total = o;
  return p;
}

__global__ __launch_bounds__(256) void k_embed_zero(uint32_t* __restrict__ p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0u;
}

// ---- fixed-point accumulation (the DETERMINISTIC mode).  Integer addition is associative, so sums
// of fixed-point values do not depend on the order in which atomics land.  Every contribution
// v = fl(+-lambda * dOut[..]) (one fp32 product, the same rounding as the atomic mode) is converted
// to a multiple of 2^-shift chosen from the largest |dOut| of the call such that |v| * 2^shift <
// 2^pbits and pbits + ceil(log2(number of chunks)) <= 62: no sum can overflow 64 bits, and the
// quantum is at least 2^-31 of the largest contribution (finer than fp32 for any realistic batch).
struct FixedScale {
  uint32_t absmax_bits;   // max over dOut of the bits of |x| (order-independent: integer max)
  uint32_t pad[3];
};

__global__ __launch_bounds__(256) void k_embed_absmax(const float* __restrict__ dOut, int64_t n,
                                                      FixedScale* __restrict__ fs) {
  // streaming read: 16-byte loads, eight of them in flight per thread (a scalar grid-stride loop was
  // latency-bound at a third of this rate); head and tail that are not 16-byte aligned go scalar
  uint32_t m = 0u;
  const int64_t tid = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t head = min(n, (int64_t)((16 - ((uintptr_t)dOut & 15)) & 15) / 4);   // floats before the first aligned one
  const int64_t nvec = (n - head) / 4;
  const vfloat4* v = reinterpret_cast<const vfloat4*>(dOut + head);
  auto take = [&](const vfloat4& x) {
    m = max(m, max(max(__float_as_uint(x.x) & 0x7fffffffu, __float_as_uint(x.y) & 0x7fffffffu),
                   max(__float_as_uint(x.z) & 0x7fffffffu, __float_as_uint(x.w) & 0x7fffffffu)));
  };
  // a workgroup takes contiguous 32 KiB pieces (8 x 256 lanes x 16 bytes), round-robin over the grid
  constexpr int U = 8;
  const int64_t piece = (int64_t)U * 256;
  for (int64_t p0 = (int64_t)blockIdx.x * piece; p0 < nvec; p0 += (int64_t)gridDim.x * piece) {
    vfloat4 x[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int64_t i = min(p0 + u * 256 + threadIdx.x, nvec - 1);      // clamped: max is idempotent
      x[u] = __builtin_nontemporal_load(v + i);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) take(x[u]);
  }
  if (tid < head) m = max(m, __float_as_uint(dOut[tid]) & 0x7fffffffu);
  const int64_t tail0 = head + 4 * nvec;
  if (tail0 + tid < n) m = max(m, __float_as_uint(dOut[tail0 + tid]) & 0x7fffffffu);
#pragma unroll
  for (int d = 32; d >= 1; d >>= 1) m = max(m, (uint32_t)__shfl_xor((int)m, d, 64));
  if ((threadIdx.x & 63) == 0 && m != 0u) atomicMax(&fs->absmax_bits, m);
}

// 2^shift as a double; NaN when dOut holds an Inf or NaN (the result is then NaN everywhere).
__device__ inline double fixed_scale(const FixedScale* fs, float lambda, int pbits) {
  const uint32_t bits = fs->absmax_bits;
  if (bits >= 0x7f800000u) return __longlong_as_double(0x7ff8000000000000ll);
  const float bound = fabsf(lambda) * __uint_as_float(bits);   // every |contribution| <= bound
  if (!(bound > 0.f)) return 1.0;
  if (!(bound < __uint_as_float(0x7f800000u))) return __longlong_as_double(0x7ff8000000000000ll);
  int ex;
  frexpf(bound, &ex);                                           // bound < 2^ex
  return ldexp(1.0, pbits - ex);
}

__device__ inline unsigned long long to_fixed(float v, double scale) {
  return (unsigned long long)__double2ll_rn((double)v * scale);
}

inline int fixed_pbits(int64_t n_items) {
  int lg = 0;
  while ((1ll << lg) < n_items + 1) ++lg;
  return 62 - lg;
}

// One thread per element: any shape, 64-bit integer atomics straight into the accumulator.
__global__ __launch_bounds__(256) void k_embed_fixed_elem(EmbedArgs a, int pbits, const int64_t* __restrict__ rows,
                                                          const uint32_t* __restrict__ tables,
                                                          const float* __restrict__ dOut, const FixedScale* fs,
                                                          unsigned long long* __restrict__ acc) {
  const int64_t e = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (e >= a.N * a.D) return;
  const double scale = fixed_scale(fs, a.lambda, pbits);
  const int64_t n = e / a.D, i = e - n * a.D, c = i / a.Z, o = i - c * a.Z;
  const int64_t off = block_offset(a.hash, tables[n], (uint64_t)rows[n], (uint64_t)c);
  const float sc = a.lambda * (float)(block_sign(a.hash, tables[n], (uint64_t)rows[n], (uint64_t)c) *
                                      elem_sign(a.hash, tables[n], (uint64_t)rows[n], (uint64_t)i));
  atomicAdd(acc + off + o, to_fixed(sc * dOut[grad_row(a, n) * a.D + i], scale));
}

__global__ __launch_bounds__(256) void k_embed_fixed_finish(int64_t m_size, float lambda, int pbits, const FixedScale* fs,
                                                            const unsigned long long* __restrict__ acc,
                                                            float* __restrict__ dM) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= m_size) return;
  const double scale = fixed_scale(fs, lambda, pbits);
  if (scale != scale) { dM[i] += __uint_as_float(0x7fc00000u); return; }
  const long long v = (long long)acc[i];
  if (v != 0) dM[i] += (float)((double)v / scale);
}

// entry = (chunk number g, key); key = offset | (negative sign << 31)
template <bool FIXED>
__global__ __launch_bounds__(kRouteThreads) void k_embed_route(EmbedArgs a, int r_log2, int nb, uint32_t cap, int walk,
                                                     const int64_t* __restrict__ rows,
                                                     const uint32_t* __restrict__ tables, uint32_t* __restrict__ cursor,
                                                     uint2* __restrict__ list, const float* __restrict__ dOut,
                                                     float* __restrict__ dM, int pbits, const FixedScale* fs,
                                                     unsigned long long* __restrict__ acc) {
  extern __shared__ __attribute__((aligned(16))) uint32_t s_route[];
  const int C = (int)a.C;
  const int rows_wg = kRouteItems / C;
  constexpr int items = kRouteItems;
  uint32_t* s_key = s_route;                                       // [items]
  uint16_t* s_pos = reinterpret_cast<uint16_t*>(s_key + items);   // [items] rank inside (workgroup, bucket)
  uint32_t* hist = s_key + items + items / 2;                      // [nb]  chunks of this workgroup per bucket
  uint32_t* gbase = hist + nb;                                     // [nb]  reserved position in the bucket's global list
  uint32_t* pre = gbase + nb;                                      // [nb]  chunks of this workgroup in the buckets before
  uint16_t* s_ord = reinterpret_cast<uint16_t*>(pre + nb);         // [items] chunk index by (bucket, rank)
  uint32_t* s_src = reinterpret_cast<uint32_t*>(s_ord + items);    // [rows_wg] gradient row of each lookup (pooled calls only)
  __shared__ uint32_t s_part[kRouteThreads];
  for (int i = threadIdx.x; i < nb; i += kRouteThreads) hist[i] = 0u;
  __syncthreads();
  const int64_t n0 = (int64_t)blockIdx.x * rows_wg;
  const int rows_here = (int)min((int64_t)rows_wg, a.N - n0);
  for (int q = threadIdx.x; q < rows_here; q += kRouteThreads) {
    const int64_t n = n0 + q;
    if (a.bag_off) s_src[q] = (uint32_t)bag_of(a.bag_off, a.B, n);
    for_each_chunk(a, walk != 0, tables[n], (uint64_t)rows[n], [&](int64_t c, int64_t off, int sgn) {
      s_key[q * C + c] = (uint32_t)off | (sgn < 0 ? 0x80000000u : 0u);
      s_pos[q * C + c] = (uint16_t)atomicAdd(&hist[(uint32_t)off >> r_log2], 1u);
    });
  }
  __syncthreads();
  // one global add per (workgroup, bucket) reserves that many consecutive list slots
  for (int i = threadIdx.x; i < nb; i += kRouteThreads) gbase[i] = hist[i] ? atomicAdd(&cursor[i], hist[i]) : 0u;
  // exclusive prefix of the histogram: where the workgroup's chunks of bucket b start when ordered
  // by (bucket, rank)
  {
    const int per = (nb + kRouteThreads - 1) / kRouteThreads;
    uint32_t sum = 0;
    for (int j = 0; j < per; ++j) {
      const int idx = threadIdx.x * per + j;
      if (idx < nb) sum += hist[idx];
    }
    s_part[threadIdx.x] = sum;
    __syncthreads();
    for (int off = 1; off < kRouteThreads; off <<= 1) {
      const uint32_t v = (int)threadIdx.x >= off ? s_part[threadIdx.x - off] : 0u;
      __syncthreads();
      s_part[threadIdx.x] += v;
      __syncthreads();
    }
    uint32_t run = s_part[threadIdx.x] - sum;
    for (int j = 0; j < per; ++j) {
      const int idx = threadIdx.x * per + j;
      if (idx < nb) { pre[idx] = run; run += hist[idx]; }
    }
  }
  __syncthreads();
  // every chunk knows its bucket and its rank inside (workgroup, bucket): that is its list slot.
  // The chunks are written out in (bucket, rank) order, so that consecutive threads store to
  // consecutive list slots of one run (a store instruction then touches a handful of lines instead
  // of 64: scattered 8-byte stores were what this kernel spent its time on).
  const int n_here = rows_here * C;
  for (int i = threadIdx.x; i < n_here; i += kRouteThreads) {
    const uint32_t b = (s_key[i] & 0x7fffffffu) >> r_log2;
    s_ord[pre[b] + s_pos[i]] = (uint16_t)i;
  }
  __syncthreads();
  for (int t = threadIdx.x; t < n_here; t += kRouteThreads) {
    const int i = s_ord[t];
    const uint32_t key = s_key[i];
    const uint32_t b = (key & 0x7fffffffu) >> r_log2;
    const uint32_t pos = gbase[b] + s_pos[i];
    // entry.x = number of the dOut chunk to add: chunk c of lookup n, or of n's bag in a pooled call
    const uint2 e = make_uint2(a.bag_off ? s_src[i / C] * (uint32_t)C + (uint32_t)(i % C) : (uint32_t)(n0 * C + i), key);
    if (pos < cap) {
      list[(size_t)b * cap + pos] = e;
    } else {
      // list full: add this chunk directly
      const float sc = (e.y & 0x80000000u) ? -a.lambda : a.lambda;
      const float* src = dOut + (int64_t)e.x * a.Z;
      if constexpr (FIXED) {
        const double scale = fixed_scale(fs, a.lambda, pbits);
        for (int o = 0; o < a.Z; ++o) atomicAdd(acc + (e.y & 0x7fffffffu) + o, to_fixed(sc * src[o], scale));
      } else {
        float* dst = dM + (e.y & 0x7fffffffu);
        for (int o = 0; o < a.Z; ++o) unsafeAtomicAdd(dst + o, sc * src[o]);
      }
    }
  }
}

template <bool FIXED>
__global__ __launch_bounds__(256) void k_embed_accum(EmbedArgs a, int r_log2, uint32_t cap, int segs_per_bucket,
                                                     const uint32_t* __restrict__ cursor, const uint2* __restrict__ list,
                                                     const float* __restrict__ dOut, float* __restrict__ dM, int pbits,
                                                     const FixedScale* fs, unsigned long long* __restrict__ acc) {
  // fp64 image: LDS fp32 atomic adds were measured ~20x slower than fp64 ones on this chip.
  // FIXED: the same 8-byte slots hold 64-bit fixed-point sums.
  using img_t = typename std::conditional<FIXED, unsigned long long, double>::type;
  extern __shared__ __attribute__((aligned(8))) char img_raw[];
  img_t* img = reinterpret_cast<img_t*>(img_raw);   // R + Z slots
  double scale = 0.0;
  if constexpr (FIXED) scale = fixed_scale(fs, a.lambda, pbits);
  const int b = blockIdx.x / segs_per_bucket, seg = blockIdx.x % segs_per_bucket;
  const uint32_t count = min(cursor[b], cap);
  const uint32_t first = (uint32_t)seg * kSeg;
  if (first >= count) return;
  const uint32_t end = min(count, first + kSeg);
  const uint2* lst = list + (size_t)b * cap;
  const int R = 1 << r_log2, span = R + a.Z;
  const int64_t slot0 = (int64_t)b << r_log2;
  for (int i = threadIdx.x; i < span; i += 256) img[i] = img_t(0);
  __syncthreads();
  const int lpi = a.Z / 4;                       // lanes per chunk
  const int ipp = 256 / lpi;                     // chunks per pass of the workgroup (Z <= 1024)
  const int sub = threadIdx.x % lpi, which = threadIdx.x / lpi;
  // Several chunks per thread in flight: the list entry and then the dOut chunk it points at are
  // dependent loads, so the entries of the next batch are fetched while this batch's chunks load.
  // The body is branch-free: a slot past the end of the list becomes chunk 0 with weight 0.
  constexpr int U = 8;
  auto add_chunk = [&](uint2 ent, vfloat4 dv) {
    const bool ok = ent.y != 0xffffffffu;
    const float sc = !ok ? 0.f : ((ent.y & 0x80000000u) ? -a.lambda : a.lambda);
    const int rel = (ok ? (int)((int64_t)(ent.y & 0x7fffffffu) - slot0) : 0) + 4 * sub;
    if constexpr (FIXED) {
      atomicAdd(&img[rel + 0], to_fixed(sc * dv.x, scale));
      atomicAdd(&img[rel + 1], to_fixed(sc * dv.y, scale));
      atomicAdd(&img[rel + 2], to_fixed(sc * dv.z, scale));
      atomicAdd(&img[rel + 3], to_fixed(sc * dv.w, scale));
    } else {
      atomicAdd(&img[rel + 0], (double)(sc * dv.x));
      atomicAdd(&img[rel + 1], (double)(sc * dv.y));
      atomicAdd(&img[rel + 2], (double)(sc * dv.z));
      atomicAdd(&img[rel + 3], (double)(sc * dv.w));
    }
  };
  if (lpi == 8) {
    // Z = 32: a pass of the workgroup takes 256 consecutive entries, one per thread, read with one
    // coalesced load; the eight lanes that serve a chunk then get its entry from the lane that
    // loaded it (lane u*8 + lane/8 of the same wave for the wave's u-th group of eight chunks).
    const int lane = threadIdx.x & 63;
    auto fetch_one = [&](uint32_t i) { return i < end ? lst[i] : make_uint2(0u, 0xffffffffu); };
    uint2 nxt = fetch_one(first + threadIdx.x);
    for (uint32_t i0 = first; i0 < end; i0 += 256) {       // uniform trip count for the workgroup
      const uint2 mine = nxt;
      uint2 e[U];
      vfloat4 d[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int src = (u * 8 + (lane >> 3)) << 2;
        e[u].x = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)mine.x);
        e[u].y = (uint32_t)__builtin_amdgcn_ds_bpermute(src, (int)mine.y);
        const uint32_t chunk = e[u].y != 0xffffffffu ? e[u].x : 0u;
        d[u] = __builtin_nontemporal_load(reinterpret_cast<const vfloat4*>(dOut + (int64_t)chunk * a.Z) + sub);
      }
      nxt = fetch_one(i0 + 256 + threadIdx.x);
#pragma unroll
      for (int u = 0; u < U; ++u) add_chunk(e[u], d[u]);
    }
  } else {
  uint2 e[U], en[U];
  auto fetch_entries = [&](uint32_t i0, uint2* dst) {
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const uint32_t i = min(i0 + u * ipp, end - 1);
      const uint2 v = lst[i];
      const bool ok = (which < ipp) && (i0 + u * ipp < end);
      dst[u] = ok ? v : make_uint2(0u, 0xffffffffu);
    }
  };
  fetch_entries(first + which, en);
  for (uint32_t i0 = first; i0 < end; i0 += U * ipp) {   // uniform trip count for the whole workgroup
#pragma unroll
    for (int u = 0; u < U; ++u) e[u] = en[u];
    vfloat4 d[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      d[u] = __builtin_nontemporal_load(reinterpret_cast<const vfloat4*>(dOut + (int64_t)e[u].x * a.Z) + sub);
    }
    fetch_entries(i0 + U * ipp + which, en);
#pragma unroll
    for (int u = 0; u < U; ++u) add_chunk(e[u], d[u]);
  }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < span; i += 256) {
    if constexpr (FIXED) {
      const unsigned long long v = img[i];
      if (v != 0ull && slot0 + i < a.m_size) atomicAdd(acc + slot0 + i, v);
    } else {
      const float v = (float)img[i];
      if (v != 0.f && slot0 + i < a.m_size) unsafeAtomicAdd(dM + slot0 + i, v);
    }
  }
}

}  // namespace

roast_status embed_fwd_launch(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, const float* M,
                              float* out, hipStream_t s) {
  return launch_embed<false>(a, rows, tables, M, out, nullptr, nullptr, s);
}

size_t embed_bucket_workspace_bytes(const EmbedArgs& a) {
  const BucketPlan p = bucket_plan(a);
  return p.ok ? p.total : 0;
}

namespace {

// route + accumulate; FIXED selects the 64-bit fixed-point variant (fs, acc in the workspace)
template <bool FIXED>
roast_status bucket_run(const EmbedArgs& a, const BucketPlan& p, const int64_t* rows, const uint32_t* tables,
                        const float* dOut, float* dM, char* base, int pbits, const FixedScale* fs,
                        unsigned long long* acc, hipStream_t s) {
  uint32_t* cursor = (uint32_t*)(base + p.cursor_off);
  uint2* list = (uint2*)(base + p.list_off);
  hipLaunchKernelGGL(k_embed_zero, dim3((p.nb + 255) / 256), dim3(256), 0, s, cursor, (int64_t)p.nb);
  const int rows_wg = kRouteItems / (int)a.C;
  const size_t lds_route = (size_t)kRouteItems * (4 + 2 + 2) + (size_t)3 * p.nb * 4 + (a.bag_off ? (size_t)rows_wg * 4 : 0);
  static std::atomic<bool> configured{false};   // per instantiation; a race between host threads only repeats the call
  if (!configured.load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_embed_route<FIXED>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024 - 8192) != hipSuccess)   // the kernel also has kRouteThreads * 4 bytes of static LDS
      return ROAST_ERR_HIP;
    // the accumulate kernel's image passes 64 KiB once buckets have 8192 slots (|M| > 8 Mi): raise
    // its limit here, before anything is launched, so that a refusal leaves dM untouched
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_embed_accum<FIXED>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (kMaxR + 1024) * 8) != hipSuccess)
      return ROAST_ERR_HIP;
    configured.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL(k_embed_route<FIXED>, dim3((unsigned)((a.N + rows_wg - 1) / rows_wg)), dim3(kRouteThreads), lds_route, s, a,
                     p.r_log2, p.nb, p.cap, walk_ok(a), rows, tables, cursor, list, dOut, dM, pbits, fs, acc);
  const int segs = (int)((p.cap + kSeg - 1) / kSeg);
  const size_t lds = ((size_t)(1 << p.r_log2) + a.Z) * 8;
  hipLaunchKernelGGL(k_embed_accum<FIXED>, dim3((unsigned)(p.nb * segs)), dim3(256), lds, s, a, p.r_log2, p.cap, segs,
                     cursor, list, dOut, dM, pbits, fs, acc);
  return hip_status(hipGetLastError());
}

inline bool bucket_worthwhile(const BucketPlan& p, const float* dOut) {
  return p.ok && p.n_items >= 65536 && ((uintptr_t)dOut & 15) == 0;
}

struct DetLayoutE {
  size_t fs_off, acc_off, bucket_off, total;
};

inline DetLayoutE det_layout_e(const EmbedArgs& a) {
  auto up = [](size_t v) { return (v + 255) / 256 * 256; };
  DetLayoutE l{};
  size_t o = 0;
  l.fs_off = o;     o += up(sizeof(FixedScale));
  l.acc_off = o;    o += up((size_t)a.m_size * 8);
  l.bucket_off = o; o += embed_bucket_workspace_bytes(a);
  l.total = o;
  return l;
}

}  // namespace

roast_status embed_bwd_atomic_launch(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables,
                                     const float* dOut, float* dM, void* ws, size_t ws_bytes, hipStream_t s) {
  const BucketPlan p = bucket_plan(a);
  // small problems, odd shapes, or no workspace: plain atomics straight into dM
  if (!bucket_worthwhile(p, dOut) || ws == nullptr || ws_bytes < p.total)
    return launch_embed<true>(a, rows, tables, nullptr, nullptr, dOut, dM, s);
  return bucket_run<false>(a, p, rows, tables, dOut, dM, (char*)ws, 0, nullptr, nullptr, s);
}

// DETERMINISTIC: largest |dOut| -> fixed-point scale; zeroed 64-bit accumulator of |M| slots in the
// workspace; the same route + accumulate pipeline (or one thread per element for the shapes it does
// not take) with integer atomics; then dM += accumulator / scale, one rounding per slot.
size_t embed_det_workspace_bytes(const EmbedArgs& a) {
  if (a.N * a.C >= (1ll << 40)) return 0;
  return det_layout_e(a).total;
}

roast_status embed_bwd_det_run(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, const float* dOut,
                               float* dM, void* ws, hipStream_t s) {
  if (a.N * a.C >= (1ll << 40)) return ROAST_ERR_UNSUPPORTED;
  const DetLayoutE l = det_layout_e(a);
  char* base = (char*)ws;
  FixedScale* fs = (FixedScale*)(base + l.fs_off);
  unsigned long long* acc = (unsigned long long*)(base + l.acc_off);
  const int pbits = fixed_pbits(a.N * a.C);
  // zero the scale record and the accumulator (contiguous: fs_off == 0, acc follows)
  const int64_t zero_words = (int64_t)((l.acc_off + (size_t)a.m_size * 8) / 4);
  const int64_t zb = (zero_words + 255) / 256;
  if (zb > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(k_embed_zero, dim3((unsigned)zb), dim3(256), 0, s, (uint32_t*)base, zero_words);
  const int64_t n_el = a.N * a.D;                               // contributions
  const int64_t n_grad = (a.bag_off ? a.B : a.N) * a.D;          // elements of dOut
  const int64_t ab = std::min<int64_t>((n_grad / 4 + 255) / 256 + 1, 256 * 8);
  hipLaunchKernelGGL(k_embed_absmax, dim3((unsigned)ab), dim3(256), 0, s, dOut, n_grad, fs);
  const BucketPlan p = bucket_plan(a);
  roast_status st;
  if (bucket_worthwhile(p, dOut)) {
    st = bucket_run<true>(a, p, rows, tables, dOut, dM, base + l.bucket_off, pbits, fs, acc, s);
  } else {
    const int64_t blocks = (n_el + 255) / 256;
    if (blocks > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_embed_fixed_elem, dim3((unsigned)blocks), dim3(256), 0, s, a, pbits, rows, tables, dOut, fs, acc);
    st = hip_status(hipGetLastError());
  }
  if (st != ROAST_OK) return st;
  hipLaunchKernelGGL(k_embed_fixed_finish, dim3((unsigned)((a.m_size + 255) / 256)), dim3(256), 0, s, a.m_size, a.lambda,
                     pbits, fs, acc, dM);
  return hip_status(hipGetLastError());
}

// ---------------------------------------------------------------------------------------------
// Lookup gradient for callers that cannot allocate: the workspace of roast_embed_bwd (bucket
// cursors and lists; in the deterministic mode also the fixed-point accumulator) lives in a
// file-scope device array instead of a caller buffer.  Every GPU the library runs on holds its own
// copy of the array, at its own address, until the process ends.
constexpr size_t kStaticScratchBytes = (size_t)64 << 20;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

namespace {
constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, once known

// Device address of this device's copy of `scratch` (in host code the array's name is only a
// stand-in for the symbol, never an address a kernel could use).
roast_status static_scratch_ptr(void** out) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return ROAST_ERR_HIP;
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return ROAST_ERR_HIP;
    g_scratch_ptr[dev].store(p, std::memory_order_release);   // a race between host threads stores the same value twice
  }
  *out = p;
  return ROAST_OK;
}
}  // namespace

size_t embed_static_scratch_bytes() { return kStaticScratchBytes; }

roast_status embed_bwd_static_run(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, const float* dOut,
                                  float* dM, bool deterministic, hipStream_t s) {
  const size_t need = deterministic ? embed_det_workspace_bytes(a) : embed_bucket_workspace_bytes(a);
  if (deterministic && need == 0) return ROAST_ERR_UNSUPPORTED;
  if (need > kStaticScratchBytes) return ROAST_ERR_WORKSPACE;
  void* ws = nullptr;
  if (need > 0) {
    const roast_status st = static_scratch_ptr(&ws);
    if (st != ROAST_OK) return st;
  }
  // From here on the device pointer `ws` stands for the array: the kernels get it as an argument,
  // exactly as they get the caller's buffer in roast_embed_bwd.  What has to start at zero (bucket
  // cursors, the fixed-point accumulator and its scale record) is cleared by fill kernels inside.
  if (deterministic) return embed_bwd_det_run(a, rows, tables, dOut, dM, ws, s);
  return embed_bwd_atomic_launch(a, rows, tables, dOut, dM, ws, need, s);
}

roast_status embed_bag_fwd_launch(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, const float* M,
                                  float* out, hipStream_t s) {
  if (a.m_size >= (1ll << 31) || a.C > kMaxC || a.hash.use_sign == 2) {
    const int64_t blocks = (a.B * a.D + 255) / 256;
    if (blocks > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
    hipLaunchKernelGGL(k_embed_bag_fwd_elem, dim3((unsigned)blocks), dim3(256), 0, s, a, rows, tables, M, out);
    return hip_status(hipGetLastError());
  }
  const bool vec4 = (a.Z % 4 == 0) && (a.D % 4 == 0) && (((uintptr_t)out & 15) == 0);
  const int64_t pieces = vec4 ? a.D / 4 : a.D;
  const int tpb = (int)std::min<int64_t>(256, pieces);      // threads per bag
  const int bags_wg = 256 / tpb;
  const int win = (int)(8192 / a.C);                        // 32 KiB of keys per window
  const int64_t blocks = (a.B + bags_wg - 1) / bags_wg;
  if (blocks > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
  const size_t lds = (size_t)win * a.C * sizeof(uint32_t);
  if (vec4)
    hipLaunchKernelGGL(k_embed_bag_fwd<4>, dim3((unsigned)blocks), dim3(256), lds, s, a, walk_ok(a), tpb, bags_wg, win,
                       rows, tables, M, out);
  else
    hipLaunchKernelGGL(k_embed_bag_fwd<1>, dim3((unsigned)blocks), dim3(256), lds, s, a, walk_ok(a), tpb, bags_wg, win,
                       rows, tables, M, out);
  return hip_status(hipGetLastError());
}

roast_status chunk_index_launch(const EmbedArgs& a, const int64_t* rows, const uint32_t* tables, int64_t* off,
                                int8_t* sgn, hipStream_t s) {
  const int64_t blocks = (a.N + 255) / 256;
  if (blocks > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(k_chunk_index, dim3((unsigned)blocks), dim3(256), 0, s, a, walk_ok(a), rows, tables, off, sgn);
  return hip_status(hipGetLastError());
}

}  // namespace roast
