// Deterministic reduction of the ROAST-MM gradient into M (gradient equation of Section 4.3 of
// arXiv 2207.10702: every slot of M receives the lambda-scaled sum of the gradients of all
// virtual weights hashed to it).
//
// Steps: (1) the tile table (offset, sign) is computed on the device and the tiles are ranked by
// (offset, tile id); (2) the per-tile products G = X^T dY are written, unscaled, to the workspace,
// one copy per I-split; (3) one thread per slot j of M walks the tiles whose interval
// [offset, offset + Z1*Z2) covers j -- a contiguous run of the ranked table because all tiles have
// the same length -- and adds their contributions in rank order, splits in index order.  No
// atomics, so the result is bit-identical from run to run.
#include "roast_internal.hpp"

namespace roast {
namespace {

constexpr int64_t kMaxTilesDet = 1 << 17;  // the ranking pass is quadratic in the number of tiles

struct DetLayout {
  size_t g_off, key_off, soff_off, order_off, sgn_off, total;
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline DetLayout det_layout(const MMArgs& a, int splits) {
  const size_t nT = (size_t)(a.nTx * a.nTy);
  DetLayout l;
  l.g_off = 0;
  l.key_off = align_up((size_t)splits * (size_t)a.H * (size_t)a.O * sizeof(float), 256);
  l.soff_off = l.key_off + align_up(nT * sizeof(int64_t), 256);
  l.order_off = l.soff_off + align_up(nT * sizeof(int64_t), 256);
  l.sgn_off = l.order_off + align_up(nT * sizeof(uint32_t), 256);
  l.total = l.sgn_off + align_up(nT * sizeof(int8_t), 256);
  return l;
}

// rank of tile t among all tiles by (offset, id); writes the sorted offsets and the permutation.
// Sixteen lanes share a tile: each counts the smaller keys among every sixteenth key of the staged
// block, and the counts are added up across the lanes (integers: any order).
constexpr int kRankLanes = 16;
__global__ __launch_bounds__(256) void k_rank_tiles(int64_t nT, const int64_t* __restrict__ off,
                                                    int64_t* __restrict__ sorted_off, uint32_t* __restrict__ order) {
  __shared__ int64_t buf[256];
  const int64_t t = ((int64_t)blockIdx.x * 256 + threadIdx.x) / kRankLanes;
  const int sub = threadIdx.x % kRankLanes;
  const int64_t mine = t < nT ? off[t] : 0;
  int rank = 0;
  for (int64_t base = 0; base < nT; base += 256) {
    const int64_t u = base + threadIdx.x;
    buf[threadIdx.x] = u < nT ? off[u] : INT64_MAX;
    __syncthreads();
    const int lim = (int)min((int64_t)256, nT - base);
    for (int q = sub; q < lim; q += kRankLanes) {
      const int64_t o = buf[q];
      rank += (o < mine || (o == mine && base + q < t)) ? 1 : 0;
    }
    __syncthreads();
  }
#pragma unroll
  for (int d = kRankLanes / 2; d >= 1; d >>= 1) rank += __shfl_xor(rank, d, 64);
  if (t < nT && sub == 0) {
    sorted_off[rank] = mine;
    order[rank] = (uint32_t)t;
  }
}

// dM[j] += sum over every virtual weight that lands on slot j, in a fixed order: the tiles that cover
// j in rank order, dealt round-robin to the eight lanes that share the slot, each lane adding its
// tiles (and their parts) in order, then a butterfly over the eight partial sums -- every level adds
// the same two values on both lanes, and fp addition is commutative, so all lanes agree bit for bit.
constexpr int kGatherLanes = 8;
__global__ __launch_bounds__(256) void k_dm_gather(MMArgs a, int splits, const float* __restrict__ G,
                                                   const int64_t* __restrict__ sorted_off,
                                                   const uint32_t* __restrict__ order, const int8_t* __restrict__ sgn,
                                                   float* __restrict__ dM) {
  const int64_t j = ((int64_t)blockIdx.x * 256 + threadIdx.x) / kGatherLanes;
  const int sub = threadIdx.x % kGatherLanes;
  const bool live = j < a.m_size;
  const int64_t nT = a.nTx * a.nTy, L = (int64_t)a.Z1 * a.Z2;
  float total = 0.f;
  int any = 0;
  if (live) {
    // first ranked tile with offset > j - L
    int64_t lo = 0, hi = nT;
    while (lo < hi) {
      const int64_t mid = (lo + hi) >> 1;
      if (sorted_off[mid] > j - L) hi = mid; else lo = mid + 1;
    }
    for (int64_t q = lo + sub; q < nT; q += kGatherLanes) {
      const int64_t o = sorted_off[q];
      if (o > j) break;
      const uint32_t t = order[q];
      const int64_t p = j - o;
      const int64_t h = (int64_t)(t / a.nTy) * a.Z1 + p / a.Z2;
      const int64_t c = (int64_t)(t % a.nTy) * a.Z2 + p % a.Z2;
      if (h >= a.H || c >= a.O) continue;
      float acc = 0.f;
      for (int s = 0; s < splits; ++s) acc += G[((int64_t)s * a.H + h) * a.O + c];
      const float es = a.hash.use_sign == 2 ? (float)elem_sign(a.hash, a.layer, (uint64_t)h, (uint64_t)c) : 1.f;
      total += a.lambda * (float)sgn[t] * es * acc;
      any = 1;
    }
  }
#pragma unroll
  for (int d = kGatherLanes / 2; d >= 1; d >>= 1) {
    total += __shfl_xor(total, d, 64);
    any |= __shfl_xor(any, d, 64);
  }
  if (live && sub == 0 && any) dM[j] += total;
}

// Sum the per-split products and scatter them: one workgroup per (tile, block of rows of the tile).
// dM[offset + Z2*o1 + o2] += lambda * sign * sum_s G[s][x*Z1 + o1][y*Z2 + o2].
// One atomic per virtual weight instead of one per weight and split.  Needs Z2 % 4 == 0, O % 4 == 0.
__global__ __launch_bounds__(256) void k_dm_scatter(MMArgs a, int splits, int rows_per_wg,
                                                    const float* __restrict__ G, float* __restrict__ dM) {
  __shared__ int64_t s_off;
  __shared__ float s_scale;
  const int chunks = (a.Z1 + rows_per_wg - 1) / rows_per_wg;
  const int64_t tile = blockIdx.x / chunks;
  const int r_begin = (blockIdx.x % chunks) * rows_per_wg;
  const int x = (int)(tile / a.nTy), y = (int)(tile % a.nTy);
  if (threadIdx.x == 0) {
    s_off = block_offset(a.hash, a.layer, (uint64_t)x, (uint64_t)y);
    s_scale = a.lambda * (float)block_sign(a.hash, a.layer, (uint64_t)x, (uint64_t)y);
  }
  __syncthreads();
  const int64_t off = s_off;
  const float scale = s_scale;
  const int n = min(rows_per_wg, a.Z1 - r_begin) * a.Z2;
  const int64_t plane = a.H * a.O;
  // Consecutive lanes take consecutive weights: the loads coalesce and each wave's atomics fall in
  // as few cache lines as possible.  The workspace is read once: non-temporal loads, the splits of
  // one element in flight together.
  for (int e = threadIdx.x; e < n; e += 256) {
    const int r = r_begin + e / a.Z2, c = e % a.Z2;
    const int64_t h = (int64_t)x * a.Z1 + r, o = (int64_t)y * a.Z2 + c;
    if (h >= a.H || o >= a.O) continue;
    const float* g = G + h * a.O + o;
    auto ld = [&](int s) { return __builtin_nontemporal_load(g + (int64_t)s * plane); };
    float acc = 0.f;
    int s = 0;
    for (; s + 8 <= splits; s += 8) {
      const float v0 = ld(s), v1 = ld(s + 1), v2 = ld(s + 2), v3 = ld(s + 3);
      const float v4 = ld(s + 4), v5 = ld(s + 5), v6 = ld(s + 6), v7 = ld(s + 7);
      acc += ((v0 + v1) + (v2 + v3)) + ((v4 + v5) + (v6 + v7));
    }
    for (; s < splits; ++s) acc += ld(s);
    unsafeAtomicAdd(dM + off + (int64_t)a.Z2 * r + c, scale * acc);
  }
}

}  // namespace

// ---- split products through the workspace, then one scatter (the fast path of the ATOMIC mode when
// the caller provides a workspace): S*H*O floats.
int dm_ws_splits(const MMArgs& a) {
  if (a.hash.use_sign == 2) return 0;   // the scatter pass applies one sign per tile
  const int s = dm_pick_splits(((a.H + 255) / 256) * ((a.O + 127) / 128), a.I, 0);   // one atomic per weight whatever s
  return s > 1 ? s : 0;               // a single split gains nothing over direct atomics
}

size_t dm_ws_workspace_bytes(const MMArgs& a) {
  const int s = dm_ws_splits(a);
  return s ? (size_t)s * (size_t)a.H * (size_t)a.O * sizeof(float) : 0;
}

roast_status dm_ws_run(const MMArgs& a, const void* X, int64_t ldx, const void* dY, int64_t ldy, float* dM, void* ws,
                       hipStream_t s) {
  const int splits = dm_ws_splits(a);
  if (!splits) return ROAST_ERR_UNSUPPORTED;
  float* G = (float*)ws;
  roast_status st = mfma_mm_bwd_dM(a, X, ldx, dY, ldy, nullptr, G, splits, s);
  if (st != ROAST_OK) return st;      // UNSUPPORTED: the caller falls back to direct atomics
  const int rows_per_wg = a.Z2 >= 1024 ? 1 : 1024 / a.Z2;    // four weights per thread
  const int chunks = (a.Z1 + rows_per_wg - 1) / rows_per_wg;
  const int64_t blocks = a.nTx * a.nTy * chunks;
  if (blocks > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(k_dm_scatter, dim3((unsigned)blocks), dim3(256), 0, s, a, splits, rows_per_wg, G, dM);
  return hip_status(hipGetLastError());
}

int dm_det_splits(const MMArgs& a) {
  // A fixed function of the shape only, so that the summation order never depends on the machine.
  const int64_t tiles = ((a.O + 255) / 256) * ((a.H + 255) / 256);
  int64_t s = (512 + tiles - 1) / tiles;
  const int64_t max_s = (a.I + 511) / 512;
  if (s > max_s) s = max_s;
  if (s > 64) s = 64;
  if (s < 1) s = 1;
  return (int)s;
}

size_t dm_det_workspace_bytes(const MMArgs& a) {
  if (a.nTx * a.nTy > kMaxTilesDet) return 0;
  return det_layout(a, dm_det_splits(a)).total;
}

roast_status dm_det_run(const MMArgs& a, roast_dtype dt, const void* X, int64_t ldx, const void* dY, int64_t ldy,
                        float* dM, void* ws, hipStream_t s) {
  const int splits = dm_det_splits(a);
  const DetLayout l = det_layout(a, splits);
  char* base = (char*)ws;
  float* G = (float*)(base + l.g_off);
  int64_t* keys = (int64_t*)(base + l.key_off);
  int64_t* soff = (int64_t*)(base + l.soff_off);
  uint32_t* order = (uint32_t*)(base + l.order_off);
  int8_t* sgn = (int8_t*)(base + l.sgn_off);
  const int64_t nT = a.nTx * a.nTy;

  roast_status st = tile_index_launch(a, keys, sgn, s);
  if (st != ROAST_OK) return st;
  hipLaunchKernelGGL(k_rank_tiles, dim3((unsigned)((nT * kRankLanes + 255) / 256)), dim3(256), 0, s, nT, keys, soff, order);
  st = hip_status(hipGetLastError());
  if (st != ROAST_OK) return st;

  st = ROAST_ERR_UNSUPPORTED;
  if (dt == ROAST_BF16) st = mfma_mm_bwd_dM(a, X, ldx, dY, ldy, nullptr, G, splits, s);
  if (st == ROAST_ERR_UNSUPPORTED) st = generic_dm_launch(a, dt, X, ldx, dY, ldy, nullptr, G, splits, s);
  if (st != ROAST_OK) return st;

  hipLaunchKernelGGL(k_dm_gather, dim3((unsigned)((a.m_size * kGatherLanes + 255) / 256)), dim3(256), 0, s, a, splits, G, soff,
                     order, sgn, dM);
  return hip_status(hipGetLastError());
}

}  // namespace roast
