// bf16 MFMA kernels for ROAST-MM on gfx950 (Algorithm 1 and the Section 4.3 gradients of
// arXiv 2207.10702): forward Y = X*W, dX = dY*W^T and the per-tile products of dM = scatter(X^T*dY),
// with W recovered from M tile by tile and never written to memory.
//
// One workgroup computes a BM x BN = 256 x 128 block of the output with specialised waves: the
// first NC waves are consumers, each owning a (BM/WGM) x (BN/WGN) sub-block in fp32 accumulators and
// doing nothing but ds_read_b128 + v_mfma_f32_32x32x16_bf16; the waves after them are producers that
// bring the next operands into LDS.  Forward / dX run sixteen waves, 128 registers per lane: eight
// consumers (two per SIMD, 64 x 64 each, so that one wave's LDS waits hide behind the other's
// MFMAs), four producers that only issue the direct-to-LDS loads of the activation operand and
// four that only stage the weight operand.  dM runs the same sixteen waves: eight consumers and
// eight producers, four transposing X and four transposing dY through registers.  The
// contraction runs in steps of BK = 64 with one workgroup barrier per step.
//
// Both operands sit in LDS as [row][k] with 128-byte rows whose 16-byte chunks are XOR-swizzled,
// so a lane fetches the 8 contraction values of its row with one conflict-free ds_read_b128
// (transposing LDS reads were measured at a quarter of that bandwidth).  How an operand gets there:
//   forward: X rows are contraction-contiguous already: global_load_lds copies them straight into
//            LDS (three stages; no registers, no ds_write), each lane fetching the chunk the swizzle
//            wants at its LDS slot.  The hashed weight tile (contiguous along O) is loaded as 8(k) x
//            4(n) register blocks, signed, rounded to bf16 and written per column (two stages);
//   dX:      dY rows likewise straight to LDS; the tile's rows run along O = the contraction, so it
//            is signed, rounded and copied row by row through registers;
//   dM:      contraction is over token rows, so X and dY are both transposed as 8 x 8 (4 x 8) bf16
//            blocks with v_perm_b32 on their way through registers (two stages each).
// Register loads run several steps ahead (one register set per step in flight); the wait counters
// are in-order, so the producer loop is branch-free and keeps one issue order, and its barriers are
// raw s_barrier instructions behind explicit s_waitcnt values (the compiler's fence would drain
// every outstanding direct-to-LDS load).
// The tile table (offset, sign) of the tiles a workgroup touches is computed by its own threads
// into LDS at kernel start.  lambda is applied to the fp32 accumulators in the epilogue, which for
// forward / dX goes through LDS (the operand stages, free by then) so that global stores are 16
// bytes per lane and row-contiguous.  Workgroups are numbered so that each XCD's L2 serves a
// contiguous band of output row blocks.
// Strips: where a launch has more blocks than CUs and few steps per block, a forward / dX workgroup
// computes several consecutive column blocks of its row block as one unbroken sequence of steps
// (Algorithm 1's loop nest seen from one workgroup: row block fixed, column blocks in turn,
// contraction innermost).  The producers never drain between blocks, the tile table is built once,
// and an inner block's accumulators leave through a small private staging area while the first
// stages of the next block are already in LDS.
#include <atomic>
#include <type_traits>
#include <utility>

#include "roast_internal.hpp"

namespace roast {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
typedef float floatx4 __attribute__((ext_vector_type(4)));
typedef uint32_t uint4v __attribute__((ext_vector_type(4)));
typedef float float4v __attribute__((ext_vector_type(4)));
typedef uint32_t uint2v __attribute__((ext_vector_type(2)));

struct __attribute__((packed, aligned(4))) f4u {  // 4 floats, 4-byte aligned (tile bases are arbitrary)
  float v[4];
};

// 4 / 8 bf16 at a 4-byte aligned address of the bf16 shadow of M.  The shadow holds two copies, the
// second shifted by one element, so that a tile base of either parity is dword-aligned in one of
// them: loads that straddle dwords were measured at three times the cost in the texture data path.
struct __attribute__((packed, aligned(4))) h4a {
  uint32_t v[2];
};
struct __attribute__((packed, aligned(4))) h8a {
  uint32_t v[4];
};

constexpr int BK = 64;
constexpr int kBM = 256, kBN = 128;   // workgroup tile of every kernel here ...
constexpr int kBNarrow = 96;          // ... but the narrow forward / dX blocks
constexpr int kMaxTable = 2048; // tile-table entries a workgroup may need
constexpr int kStripTable = 768; // ... when it computes a strip of blocks: the table's tail then stages the strip's inner blocks
enum { MODE_FWD = 0, MODE_DX = 1, MODE_DM = 2 };

__device__ inline uint32_t pack_bf16x2(float a, float b) {
  typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
  bf16x2 r = {(__bf16)a, (__bf16)b};
  return __builtin_bit_cast(uint32_t, r);
}

// s_waitcnt immediate (gfx9 layout: vmcnt in bits 3:0 and 15:14, expcnt 6:4, lgkmcnt 11:8) that
// waits until at most n vector-memory operations are outstanding and leaves the other counters alone.
constexpr int vmcnt_only(int n) { return (n & 15) | ((n >> 4) << 14) | 0x0f70; }

// Byte offset of 16-byte chunk `chunk` (0..7) of row `row` inside an operand tile.
__device__ inline int lds_off(int row, int chunk) {
  return row * 128 + (((chunk ^ row ^ (row >> 3)) & 7) << 4);
}

struct KernArgs {
  MMArgs a;
  const uint16_t* A;   // FWD: X, DX: dY, DM: X
  int64_t lda;
  const uint16_t* B;   // DM: dY
  int64_t ldb;
  const float* M;      // FWD / DX
  const uint16_t* Mb;  // FWD / DX: bf16 shadow of M (SHADOW kernels): copy 0, and copy 1 (shifted by one) at +mb_stride
  int64_t mb_stride;
  uint16_t* C;         // FWD: Y, DX: dX
  int64_t ldc;
  // X3 kernels (fp32 operands split into three bfloat16 planes): element distance between the planes
  // of A, of B (dM only) and of the shadow of M, and the fp32 output of FWD / DX (row stride ldc)
  int64_t a_plane, b_plane, mb_plane;
  float* C32;
  float* dM;           // DM, atomic mode
  float* G;            // DM, deterministic mode: raw products [split][H][O]
                       // FWD / DX with a split contraction: fp32 partial outputs [split][I][columns]
  int rows_per_split;  // length of one part of the contraction axis (DM always; FWD / DX when nbz > 1)
  int split_begin[18]; // dM with uneven parts (all zero: unused): part z covers rows [split_begin[z], split_begin[z+1])
  int nbx, nby, nbz;   // logical block grid: columns (x), rows (y), contraction splits (z)
  // Forward / dX strips: a workgroup computes `ntile` consecutive column blocks one after the other
  // as one continuous sequence of contraction steps (1 = one block per workgroup); consecutive
  // blocks of a strip are `tile_shift` = BN / Z hash tiles apart.
  int ntile, tile_shift;
  // log2 of Z1 / Z2 when they are powers of two, else -1 (set by launch()): the per-step tile lookups
  // of the load waves and the dM epilogue then shift and mask instead of dividing
  int z1_shift, z2_shift;
};

// v / z and v % z for v >= 0: a shift and a mask when z is a power of two (sh = log2 z), the division
// otherwise.  sh is uniform, so this is a scalar branch around ~25 instructions per division.
__device__ inline int tile_div(int v, int z, int sh) {
  if (sh >= 0) return v >> sh;
  return v / z;
}
__device__ inline int tile_mod(int v, int z, int sh) {
  if (sh >= 0) return v & (z - 1);
  return v % z;
}

// Workgroups are handed to the 8 XCDs round-robin, and each XCD has its own L2.  Blocks that share
// an operand slab (same row block -> same rows of X / dY) should therefore run on the same XCD:
// XCD j takes the j-th contiguous eighth of the row-major block order (z, y, x), so that an operand
// slab is fetched into one L2 and reused there by all the column blocks, instead of being fetched by
// eight L2s from the memory-side cache.  Returns false for the padding workgroups of the last eighth.
__device__ inline bool block_coords(const KernArgs& p, int* bx, int* by, int* bz) {
  const int total = p.nbx * p.nby * p.nbz;
  const int chunk = (total + 7) / 8;
  const int w = blockIdx.x;
  const int t = (w & 7) * chunk + (w >> 3);
  if ((w >> 3) >= chunk || t >= total) return false;
  *bx = t % p.nbx;
  *by = (t / p.nbx) % p.nby;
  *bz = t / (p.nbx * p.nby);
  return true;
}

// Transposing loaders for a bf16 [BK rows (k)][W cols] tile whose rows are contiguous in memory, one
// per tile width, both with 16-byte loads (a wave's vector-memory instructions issue slowly next to
// busy consumers, so a step's bytes should come in as few of them as possible: with 8-byte loads for
// the 128-wide tile the dM product took 3-5 % longer).
// 256 columns: each thread owns an 8(k) x 8(cols) block, loads its 8 row pieces, and writes 8 16-byte
// chunks (8 k-values of one column) to the [col][k] LDS tile.
template <int W>
struct TLoad {
  static_assert(W == 256, "the 128-column tile has its own loader");
  static constexpr int KB_SHIFT = 5, COL_MASK = 31;   // thread -> column block ptid & 31 (8 columns), k-block ptid >> 5 (8 rows)
  static constexpr int COLS = 8;                      // columns per thread
  uint32_t r[8][4];
  __device__ void load(const uint16_t* src, int64_t ld, int k0, int kmax_row, int col, int kb) {
    // (both paths issue the same eight loads in the same order; the branch is uniform: only a
    // step that reaches past the last row has to clamp its row numbers)
    if (k0 + BK - 1 <= kmax_row) {
      const uint16_t* p0 = src + (int64_t)(k0 + 8 * kb) * ld + col;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const uint4v v = *reinterpret_cast<const uint4v*>(p0 + (int64_t)q * ld);
        r[q][0] = v[0]; r[q][1] = v[1]; r[q][2] = v[2]; r[q][3] = v[3];
      }
    } else {
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int row = min(k0 + 8 * kb + q, kmax_row);
        const uint4v v = *reinterpret_cast<const uint4v*>(src + (int64_t)row * ld + col);
        r[q][0] = v[0]; r[q][1] = v[1]; r[q][2] = v[2]; r[q][3] = v[3];
      }
    }
  }
  // rows at or beyond k_end are zeroed (they would add into sums that are kept); only the last step
  // of a contraction part can have any (uniform branch)
  __device__ void store(char* tile, int k0, int k_end, int colblk, int kb) {
    if (k0 + BK > k_end) {
#pragma unroll
      for (int q = 0; q < 8; ++q)
        if (k0 + 8 * kb + q >= k_end) {
#pragma unroll
          for (int d = 0; d < 4; ++d) r[q][d] = 0u;
        }
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
      uint4v o;
#pragma unroll
      for (int pr = 0; pr < 4; ++pr) o[pr] = __builtin_amdgcn_perm(r[2 * pr + 1][c >> 1], r[2 * pr][c >> 1], sel);
      *reinterpret_cast<uint4v*>(tile + lds_off(colblk * 8 + c, kb)) = o;
    }
  }
};
// 128 columns: each thread owns a 4(k) x 8(cols) block, loads its 4 row pieces, and writes 8 half
// chunks (4 k-values of one column, 8 bytes).
template <>
struct TLoad<128> {
  static constexpr int KB_SHIFT = 4, COL_MASK = 15;   // thread -> column group ptid & 15 (8 columns), k-block ptid >> 4 (4 rows)
  static constexpr int COLS = 8;
  uint32_t r[4][4];
  __device__ void load(const uint16_t* src, int64_t ld, int k0, int kmax_row, int col, int kb) {
    if (k0 + BK - 1 <= kmax_row) {
      const uint16_t* p0 = src + (int64_t)(k0 + 4 * kb) * ld + col;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const uint4v v = *reinterpret_cast<const uint4v*>(p0 + (int64_t)q * ld);
        r[q][0] = v[0]; r[q][1] = v[1]; r[q][2] = v[2]; r[q][3] = v[3];
      }
    } else {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int row = min(k0 + 4 * kb + q, kmax_row);
        const uint4v v = *reinterpret_cast<const uint4v*>(src + (int64_t)row * ld + col);
        r[q][0] = v[0]; r[q][1] = v[1]; r[q][2] = v[2]; r[q][3] = v[3];
      }
    }
  }
  __device__ void store(char* tile, int k0, int k_end, int colblk, int kb) {
    if (k0 + BK > k_end) {
#pragma unroll
      for (int q = 0; q < 4; ++q)
        if (k0 + 4 * kb + q >= k_end) {
#pragma unroll
          for (int d = 0; d < 4; ++d) r[q][d] = 0u;
        }
    }
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const uint32_t sel = (c & 1) ? 0x07060302u : 0x05040100u;
      const uint2v o = {__builtin_amdgcn_perm(r[1][c >> 1], r[0][c >> 1], sel),
                        __builtin_amdgcn_perm(r[3][c >> 1], r[2][c >> 1], sel)};
      *reinterpret_cast<uint2v*>(tile + lds_off(colblk * 8 + c, kb >> 1) + 8 * (kb & 1)) = o;
    }
  }
};

// ---------------------------------------------------------------------------------------------
// Producer side: per-thread addressing context and one register set of staged operand data.
template <int MODE, int BM, int BN>
struct ProdCtx {
  static constexpr int A_LOADS = BM / 32;     // direct-to-LDS instructions per producer wave and step
  static constexpr int FW_NG = BN / 4, FW_KBS = 256 / FW_NG, FW_BLK = 8 / FW_KBS;
  static constexpr int DX_LOADS = BN / 32;
  int ptid;
  // FWD / DX, A operand: source of this lane for each of the wave's direct-to-LDS loads
  const uint16_t* a_ptr[MODE == MODE_DM ? 1 : A_LOADS];
  // FWD, B operand: 8(k) x 4(n) fp32 blocks; thread -> column group ptid % FW_NG, k-blocks ptid / FW_NG + FW_KBS*b
  int fw_yl, fw_nin;
  // FWD from the bf16 shadow: 4(k) x 8(n) bf16 blocks (16-byte loads); thread -> column group ptid % FS_NG, k-block ptid / FS_NG
  static constexpr int FS_NG = BN / 8;
  static_assert(FS_NG <= 16, "at most one 4 x 8 block per producer thread and 64-deep step (threads beyond 16 * FS_NG idle)");
  int fs_yl, fs_nin;
  // DX, B operand: BN rows (h) x 8 chunks of 8 floats; thread -> chunk (ptid & 7) of rows (ptid >> 3) + 32*q
  int dx_ent[MODE == MODE_DX ? DX_LOADS : 1];
  int dx_rowoff[MODE == MODE_DX ? DX_LOADS : 1];
  // DM: 8(k) x 8 blocks of X, 4(k) x 8 blocks of dY (TLoad<256>, TLoad<128>): first column of this thread's block
  int ta_col, tb_col;
  // ELEM (forward / dX, one hash per virtual weight): thread -> LDS row ptid & 127 (one output
  // column: the "fixed" coordinate) and half ptid >> 7 of the 64-deep step (32 consecutive values of
  // the contraction index: the "running" coordinate).  el_u / el_s: the fixed coordinate's part of
  // the offset hash and of the sign hash; el_inner: its part of the offset inside the tile.
  uint32_t el_u, el_s;
  int el_inner;
};

// f(integral_constant<int, 0>) ... f(integral_constant<int, N - 1>): a loop whose index is a constant expression
template <typename F, int... Is>
__device__ inline void static_for_impl(F&& f, std::integer_sequence<int, Is...>) {
  (f(std::integral_constant<int, Is>{}), ...);
}
template <int N, typename F>
__device__ inline void static_for(F&& f) {
  static_for_impl(f, std::make_integer_sequence<int, N>{});
}

// (a + b) mod P for a, b < P < 2^32
__device__ inline uint32_t addmod32(uint32_t a, uint32_t b, uint32_t P) {
  const uint32_t s = a + b;
  return (s < a || s >= P) ? s - P : s;
}

template <int MODE, int BM, int BN, bool SHADOW>
struct RegSet {
  using Ctx = ProdCtx<MODE, BM, BN>;
  // weight tile from fp32 M ...
  floatx4 fw_reg[(MODE == MODE_FWD && !SHADOW) ? Ctx::FW_BLK * 8 : 1];
  float fw_sgn;
  floatx4 dx_reg[(MODE == MODE_DX && !SHADOW) ? Ctx::DX_LOADS * 2 : 1];
  float dx_sgn[MODE == MODE_DX ? Ctx::DX_LOADS : 1];
  // ... or from its bf16 shadow
  uint4v fs_reg[(MODE == MODE_FWD && SHADOW) ? 4 : 1];
  uint4v ds_reg[(MODE == MODE_DX && SHADOW) ? Ctx::DX_LOADS : 1];
};

// ELEM: 32 gathered weights of one output column and one bit of sign each
struct ElemRegs {
  float w[32];
  uint32_t neg;
};


// X3: fp32 in, fp32 out on the bf16 matrix cores.  Every fp32 operand value x is held as three
// bfloat16 planes with x = hi + mid + lo exactly (3 x 8 significand bits); a product x*w is the sum
// of nine plane products, of which the six of weight >= 2^-16 are kept: (hi,hi) (hi,mid) (mid,hi)
// (hi,lo) (lo,hi) (mid,mid).  The planes are truncated (|mid| < 2^-7 |x|, |lo| < 2^-14 |x|), so the
// three dropped products are bounded by 2^-21 |x||w| per term in the worst case (mid and lo planes
// all ones) and are near 2^-24 |x||w| for typical mantissas; the accumulation is the usual fp32 one.  The contraction loop simply runs six times as many steps: step = 6*kq + pair.
// RAGK: the contraction length of forward / dX is a multiple of 8 but not of 64 (a separate
// instantiation: the extra selects in the load waves cost the regular kernels 15 %).
// ELEM: one hash per virtual weight instead of one per tile.  Forward / dX: the weight producers
// gather every element of their 64 x 128 slab of W from M through the hash (any tile size down to
// 1 x 1, per-tile or per-element sign), round it and stage it like the tiled kernels do, so the same
// consumers run; dM: the epilogue hashes every accumulator element to its slot.  This is the
// element-wise (HashedNet-style) map of Section 3 run at the same arithmetic as the tiled map.
template <int MODE, int BM, int BN, int WGM, int WGN, bool SHADOW, bool X3 = false, bool RAGK = false, bool ELEM = false>
__global__ __launch_bounds__((WGM * WGN + 8) * 64) void k_roast_mfma(KernArgs p) {
  static_assert(!X3 || SHADOW || MODE == MODE_DM, "the plane kernels read the weight planes, not fp32 M");
  static_assert(!ELEM || (!SHADOW && !X3 && BN == 128 && (RAGK || MODE == MODE_DM)), "element-wise staging: fp32 M, 128-wide blocks, any contraction length");
  constexpr int NC = WGM * WGN;                  // consumer waves
  // Eight producer waves follow the consumers: waves NC..NC+3 bring in the A operand (forward / dX:
  // direct-to-LDS loads of the activations; dM: X transposed through registers), waves NC+4..NC+7
  // the B operand (weight tile; dM: dY transposed).  A wave's vector-memory instructions were
  // measured to issue more than 100 cycles apart next to busy consumers, so the loads of a step are
  // spread over eight waves rather than four.
  constexpr int NPW = 8;
  constexpr int NT = (NC + NPW) * 64;            // threads of the workgroup
  static_assert(NC == 4 || NC == 8, "one or two consumer waves per SIMD");
  using Ctx = ProdCtx<MODE, BM, BN>;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;  // consumer wave tile
  constexpr int MI = WTM / 32, NI = WTN / 32;    // 32x32 blocks per wave
  constexpr int A_BYTES = BM * 128, B_BYTES = BN * 128;
  constexpr int EPI_STRIDE = WTN * 2 + 16;       // bytes per row of a wave's epilogue buffer
  constexpr int EPI_BYTES = NC * 32 * EPI_STRIDE; // aliases the operand stages once the contraction is done
  // Forward / dX: the activation operand needs no conversion, so it goes from global memory
  // straight into LDS (global_load_lds, no registers, no ds_write) through three stages; the weight
  // operand and both operands of dM pass through registers into two stages.
  constexpr bool ADMA = (MODE != MODE_DM);
  constexpr int NA = ADMA ? 3 : 2;               // LDS stages of the A operand
  constexpr int TILES_BYTES = NA * A_BYTES + 2 * B_BYTES;

  extern __shared__ __attribute__((aligned(1024))) char smem[];
  static_assert(EPI_BYTES <= TILES_BYTES, "epilogue staging must fit in the operand stages");
  int64_t* s_off = reinterpret_cast<int64_t*>(smem + TILES_BYTES);
  float* s_sgn = reinterpret_cast<float*>(smem + TILES_BYTES + kMaxTable * 8);
  auto a_stage = [&](int step) -> char* { return smem + (step % NA) * A_BYTES; };
  auto b_stage = [&](int step) -> char* { return smem + NA * A_BYTES + (step & 1) * B_BYTES; };

  const MMArgs& a = p.a;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool producer = wave >= NC;
  const int I = (int)a.I;
  int bx, by, bz;
  if (!block_coords(p, &bx, &by, &bz)) return;   // whole workgroup leaves before any barrier
  const int NTL = MODE == MODE_DM ? 1 : max(p.ntile, 1);     // column blocks of this workgroup's strip
  const int m0 = by * BM, n0 = bx * BN * NTL;                // n0: first column of the strip
  const int Mdim = MODE == MODE_DM ? (int)a.H : I;
  const int Ndim = MODE == MODE_DX ? (int)a.H : (int)a.O;
  int k_begin = 0, k_end = MODE == MODE_FWD ? (int)a.H : (MODE == MODE_DX ? (int)a.O : I);
  if (MODE == MODE_DM || p.nbz > 1) {
    if (MODE == MODE_DM && p.split_begin[1] > 0) {
      k_begin = p.split_begin[bz];
      k_end = p.split_begin[bz + 1];
    } else {
      k_begin = bz * p.rows_per_split;
      k_end = min(k_end, k_begin + p.rows_per_split);
    }
  }
  const int nsteps_k = max(0, (k_end - k_begin + BK - 1) / BK);
  // A strip runs its blocks back to back: step s belongs to block s / nsteps_k and to contraction
  // step s % nsteps_k of it, so the producers never drain between two blocks of a strip.
  const int nsteps = X3 ? 6 * nsteps_k : nsteps_k * NTL;         // identical for every wave of the workgroup
  const int nk1 = max(nsteps_k, 1);
  auto step_k0 = [&](int step) { return k_begin + (X3 ? step / 6 : (NTL == 1 ? step : step % nk1)) * BK; };
  auto step_shift = [&](int step) { return NTL == 1 ? 0 : (step / nk1) * p.tile_shift; };   // hash tiles between block 0 and the step's block
  auto step_asel = [&](int step) { return X3 ? (0x120100 >> (4 * (step % 6))) & 3 : 0; };   // plane of A
  auto step_bsel = [&](int step) { return X3 ? (0x102010 >> (4 * (step % 6))) & 3 : 0; };   // plane of B / M

  // ---- tile table (all threads but the waves that only issue direct-to-LDS loads: those have the
  // first step's loads on their way while the others hash, and meet them at the barrier below)
  // FWD: entry [kt * TN + yl] for tile (x = kt, y = n0/Z2 + yl), TN = tiles spanned by BN along O
  // DX : entry [kt * TN + xl] for tile (x = n0/Z1 + xl, y = kt), TN = tiles spanned by BN along H
  // DM : entry [xl * TN + yl] for tile (x = m0/Z1 + xl, y = n0/Z2 + yl)
  int TN = 1;
  const bool dma_wave = ADMA && wave >= NC && wave < NC + 4;
  {
    int x0 = 0, y0 = 0, cnt = 0;
    if (MODE == MODE_FWD) {
      y0 = n0 / a.Z2;
      TN = (min(n0 + BN * NTL, (int)a.O) - 1) / a.Z2 - y0 + 1;
      cnt = (int)a.nTx * TN;
    } else if (MODE == MODE_DX) {
      x0 = n0 / a.Z1;
      TN = (min(n0 + BN * NTL, (int)a.H) - 1) / a.Z1 - x0 + 1;
      cnt = (int)a.nTy * TN;
    } else {
      x0 = m0 / a.Z1; y0 = n0 / a.Z2;
      TN = (min(n0 + BN, (int)a.O) - 1) / a.Z2 - y0 + 1;
      cnt = ((min(m0 + BM, (int)a.H) - 1) / a.Z1 - x0 + 1) * TN;
    }
    constexpr int NB = ADMA ? NT - 256 : NT;     // threads that build the table
    const int bi = (ADMA && wave >= NC) ? tid - 256 : tid;
    if (ELEM) cnt = 0;                           // no tile table: every element is hashed where it is used
    for (int e = dma_wave ? cnt : bi; e < cnt; e += NB) {
      uint64_t x, y;
      if (MODE == MODE_FWD) { x = e / TN; y = y0 + e % TN; }
      else if (MODE == MODE_DX) { y = e / TN; x = x0 + e % TN; }
      else { x = x0 + e / TN; y = y0 + e % TN; }
      s_off[e] = block_offset(a.hash, a.layer, x, y);
      s_sgn[e] = (float)block_sign(a.hash, a.layer, x, y);
    }
  }
  if (!dma_wave) __syncthreads();

  if (producer) {
    // =========================================================================== producer waves
    // Loads are unconditional: rows / columns outside the problem are redirected to a valid address
    // and their products are never stored; only the contraction tail of the dM product is zeroed.
    // The producers' instructions are few but on the critical path of every step; with equal
    // priority the SIMD's arbiter favours the consumer waves and the producer only runs while they
    // sit at the barrier (measured: the two phases then serialise).
    // The waves that only issue direct-to-LDS loads have nothing on the critical path but the wait
    // for their loads: they stay at the default priority (raising it too cost 4-8 %).
    if (!(MODE != MODE_DM && wave < NC + 4)) __builtin_amdgcn_s_setprio(3);
    Ctx c;
    constexpr int B_WAVE0 = NC + 4;                // first wave that stages the B operand
    const bool a_role = wave < B_WAVE0;
    const bool a_producer = ADMA && a_role;        // issues direct-to-LDS loads only
    c.ptid = a_role ? tid - NC * 64 : tid - B_WAVE0 * 64;
    const int pt = c.ptid;
    // A operand: producer wave w copies rows w*BM/4 .. +BM/4 of the tile, 8 rows per instruction.
    // A direct-to-LDS load puts lane l's 16 bytes at (LDS base) + 16*l, i.e. row l/8, physical chunk
    // l%8 of that 8-row group -- so the lane fetches the logical chunk the XOR swizzle keeps there.
    if (a_producer) {
#pragma unroll
      for (int q = 0; q < Ctx::A_LOADS; ++q) {
        const int r = (wave - NC) * (BM / 4) + q * 8 + (lane >> 3);
        const int ch = (lane ^ r ^ (r >> 3)) & 7;
        c.a_ptr[q] = p.A + (int64_t)min(m0 + r, I - 1) * p.lda + 8 * ch;
      }
    }
    // Always issued (a step past the end is clamped and lands in a stage nobody reads any more), so
    // that the in-order wait counts below are the same in every iteration.
    auto dma_issue = [&](int step) {
      if constexpr (ADMA) {
        const int st = min(step, nsteps - 1);
        const int kk = step_k0(st);
        const int64_t pl = X3 ? step_asel(st) * p.a_plane : 0;
        char* dst = a_stage(step) + (wave - NC) * (BM / 4) * 128;
        // A ragged contraction length (a multiple of 8, not of 64): the 16-byte pieces of the last
        // step that lie beyond it are fetched from the start of the row instead (any finite value
        // will do: the weight rows they meet are staged as zeros).  ch(q) = ch(0) ^ q, see above.
        const bool ragged = RAGK && kk + BK > k_end;
        const int ch0 = (lane ^ (lane >> 3)) & 7;
#pragma unroll
        for (int q = 0; q < Ctx::A_LOADS; ++q) {
          const int ch8 = 8 * (ch0 ^ (q & 7));
          const int64_t koff = (RAGK && ragged && kk + ch8 >= k_end) ? pl - ch8 : pl + kk;
          __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void*)(c.a_ptr[q] + koff),
                                           (__attribute__((address_space(3))) void*)(dst + q * 1024), 16, 0, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    };
    if (MODE == MODE_FWD) {
      const int n = min(n0 + 4 * (pt % Ctx::FW_NG), (int)a.O - 4);
      c.fw_yl = n / a.Z2 - n0 / a.Z2;
      c.fw_nin = n % a.Z2;
      const int n8 = min(n0 + 8 * (pt % Ctx::FS_NG), (int)a.O - 8);
      c.fs_yl = n8 / a.Z2 - n0 / a.Z2;
      c.fs_nin = n8 % a.Z2;
    }
    if (MODE == MODE_DX) {
#pragma unroll
      for (int q = 0; q < Ctx::DX_LOADS; ++q) {
        const int h = min(n0 + (pt >> 3) + 32 * q, (int)a.H - 1);
        c.dx_ent[q] = h / a.Z1 - n0 / a.Z1;
        c.dx_rowoff[q] = a.Z2 * (h % a.Z1);
      }
    }
    if constexpr (MODE == MODE_DM) {
      c.ta_col = min(m0 + (pt & TLoad<BM>::COL_MASK) * TLoad<BM>::COLS, (int)a.H - TLoad<BM>::COLS);
      c.tb_col = min(n0 + (pt & TLoad<BN>::COL_MASK) * TLoad<BN>::COLS, (int)a.O - TLoad<BN>::COLS);
    }
    // ELEM.  W[i, j] sits at offset(x, y) + Z2 * (i mod Z1) + (j mod Z2), x = i / Z1, y = j / Z2, with
    // sign g(x, y) or g(i, j).  The hash of a key is a sum of per-coordinate terms mod P, so a thread
    // keeps the terms of its fixed coordinate (forward: j = its output column; dX: i = its output
    // column) and walks the running coordinate (the contraction index) with adds.
    constexpr bool EL_FWD = MODE == MODE_FWD;
    const uint32_t el_P = (uint32_t)a.hash.P.d;
    const int el_zrun = EL_FWD ? a.Z1 : a.Z2;                                  // tile extent along the running coordinate
    const uint32_t el_ca = (uint32_t)(EL_FWD ? a.hash.a1 : a.hash.a2);         // offset-hash coefficient of the running tile index
    const uint32_t el_cs = (uint32_t)(EL_FWD ? a.hash.s1 : a.hash.s2);         // sign-hash coefficient of the running index
    if constexpr (ELEM && MODE != MODE_DM) {
      const int f = min(n0 + (pt & 127), Ndim - 1);
      const int zf = EL_FWD ? a.Z2 : a.Z1;
      const uint64_t tf = (uint64_t)(f / zf), L = bmod(a.layer, a.hash.P);
      c.el_u = (uint32_t)bmod(bmod(a.hash.a0 * L, a.hash.P) + bmod((EL_FWD ? a.hash.a2 : a.hash.a1) * tf, a.hash.P) + a.hash.a3,
                              a.hash.P);
      const uint64_t sk = a.hash.use_sign == 2 ? (uint64_t)f : tf;             // element sign: keyed by the coordinate itself
      c.el_s = (uint32_t)bmod(bmod(a.hash.s0 * L, a.hash.P) + bmod((EL_FWD ? a.hash.s2 : a.hash.s1) * sk, a.hash.P) + a.hash.s3,
                              a.hash.P);
      c.el_inner = EL_FWD ? f % zf : a.Z2 * (f % zf);
    }
    [[maybe_unused]] auto elem_load = [&](ElemRegs& r, int step) {
      const int t0 = step_k0(step) + 32 * (pt >> 7);                           // first running index of this thread
      const int tile0 = t0 / el_zrun;
      int rem = t0 - tile0 * el_zrun;
      uint32_t run_u = (uint32_t)bmod((uint64_t)el_ca * (uint64_t)tile0, a.hash.P);
      uint32_t run_s = a.hash.use_sign == 0 ? 0u
                       : (uint32_t)bmod((uint64_t)el_cs * (uint64_t)(a.hash.use_sign == 2 ? t0 : tile0), a.hash.P);
      const int inner_mul = EL_FWD ? a.Z2 : 1;
      uint32_t neg = 0u;
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int e = 0; e < 32; ++e) {
        const uint32_t u = addmod32(c.el_u, run_u, el_P);
        const int64_t idx = (int64_t)((uint64_t)a.hash.align * mod_slots32(a.hash, u)) + c.el_inner + inner_mul * rem;
        r.w[e] = p.M[(t0 + e < k_end) ? idx : 0];                              // beyond the contraction: any valid slot, zeroed below
        if (a.hash.use_sign != 0) neg |= (addmod32(c.el_s, run_s, el_P) & 1u) << e;
        ++rem;
        const bool wrap = rem == el_zrun;
        rem = wrap ? 0 : rem;
        run_u = wrap ? addmod32(run_u, el_ca, el_P) : run_u;
        if (a.hash.use_sign == 2 || (a.hash.use_sign == 1 && wrap)) run_s = addmod32(run_s, el_cs, el_P);
      }
      r.neg = neg;
      __builtin_amdgcn_sched_barrier(0);
    };
    [[maybe_unused]] auto elem_store = [&](ElemRegs& r, int step) {
      char* Bt = b_stage(step);
      const int t0 = step_k0(step) + 32 * (pt >> 7);
#pragma unroll
      for (int cc = 0; cc < 4; ++cc) {
        uint4v o;
#pragma unroll
        for (int pr = 0; pr < 4; ++pr) {
          const int e0 = 8 * cc + 2 * pr;
          float v0 = (r.neg >> e0) & 1u ? -r.w[e0] : r.w[e0];
          float v1 = (r.neg >> (e0 + 1)) & 1u ? -r.w[e0 + 1] : r.w[e0 + 1];
          if (t0 + e0 >= k_end) v0 = 0.f;
          if (t0 + e0 + 1 >= k_end) v1 = 0.f;
          o[pr] = pack_bf16x2(v0, v1);
        }
        *reinterpret_cast<uint4v*>(Bt + lds_off(pt & 127, 4 * (pt >> 7) + cc)) = o;
      }
    };

    auto load_global = [&](RegSet<MODE, BM, BN, SHADOW>& r, int step) {
      const int k0 = step_k0(step);
      [[maybe_unused]] const uint16_t* Mb = X3 ? p.Mb + step_bsel(step) * p.mb_plane : p.Mb;
      // Keep the issue order of the load groups the same everywhere (prologue and loop): the wait
      // counters are in-order, and a differing order would make the waits before the LDS writes
      // cover the newest loads as well.
      __builtin_amdgcn_sched_barrier(0);
      if (MODE == MODE_FWD && SHADOW) {
        // this thread's 4 k-rows lie in one hash tile (Z1 % 4 == 0), not necessarily the step's first
        // (a block narrower than 128 columns leaves the threads beyond 16 * FS_NG without work:
        // they repeat the last row block's loads and store nothing)
        const int kraw = k0 + 4 * min(pt / Ctx::FS_NG, 15);
        const int kabs = RAGK ? min(kraw, k_end - 4) : kraw;   // rows beyond a ragged contraction length: zeros below
        const int e = tile_div(kabs, a.Z1, p.z1_shift) * TN + c.fs_yl + step_shift(step);
        const int64_t off0 = s_off[e];
        const int64_t rel = off0 + (int64_t)a.Z2 * tile_mod(kabs, a.Z1, p.z1_shift) + c.fs_nin;
        // everything added to the tile base is even (Z2 % 8 == 0): the base's parity picks the copy
        const uint16_t* mb = Mb + ((off0 & 1) ? p.mb_stride - 1 : 0);
        r.fw_sgn = s_sgn[e];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          const h8a m = *reinterpret_cast<const h8a*>(mb + rel + (int64_t)q * a.Z2);
          r.fs_reg[q] = (!RAGK || kraw < k_end) ? uint4v{m.v[0], m.v[1], m.v[2], m.v[3]} : uint4v{0u, 0u, 0u, 0u};
        }
      } else if (MODE == MODE_FWD) {
        static_assert(MODE != MODE_FWD || SHADOW || Ctx::FW_BLK == 1, "one 8-row block per thread: one tile, one sign");
        const int kraw = k0 + 8 * (pt / Ctx::FW_NG);   // 8 k-rows in one hash tile (Z1 % 8 == 0)
        const int kabs = RAGK ? min(kraw, k_end - 8) : kraw;
        const int e = tile_div(kabs, a.Z1, p.z1_shift) * TN + c.fw_yl + step_shift(step);
        const int64_t rel = s_off[e] + (int64_t)a.Z2 * tile_mod(kabs, a.Z1, p.z1_shift) + c.fw_nin;
        r.fw_sgn = s_sgn[e];
#pragma unroll
        for (int b = 0; b < Ctx::FW_BLK; ++b)
#pragma unroll
          for (int q = 0; q < 8; ++q) {
            const int64_t at = rel + (int64_t)(8 * Ctx::FW_KBS * b + q) * a.Z2;
            const f4u m = *reinterpret_cast<const f4u*>(p.M + at);
            r.fw_reg[b * 8 + q] = (!RAGK || kraw < k_end) ? floatx4{m.v[0], m.v[1], m.v[2], m.v[3]} : floatx4{0.f, 0.f, 0.f, 0.f};
          }
      } else if (MODE == MODE_DX && SHADOW) {
        // this thread's 8-wide chunk of the contraction axis lies in one hash tile (Z2 % 8 == 0)
        const int kraw = k0 + 8 * (pt & 7);
        const int kabs = RAGK ? min(kraw, k_end - 8) : kraw;   // chunks beyond a ragged contraction length: zeros
        const int kt = tile_div(kabs, a.Z2, p.z2_shift) * TN + step_shift(step), kin = tile_mod(kabs, a.Z2, p.z2_shift);
#pragma unroll
        for (int q = 0; q < Ctx::DX_LOADS; ++q) {
          const int e = kt + c.dx_ent[q];
          const int64_t off0 = s_off[e];
          const uint16_t* mb = Mb + ((off0 & 1) ? p.mb_stride - 1 : 0);     // row offsets are even (Z2 % 8 == 0)
          const h8a m = *reinterpret_cast<const h8a*>(mb + off0 + c.dx_rowoff[q] + kin);
          r.ds_reg[q] = (!RAGK || kraw < k_end) ? uint4v{m.v[0], m.v[1], m.v[2], m.v[3]} : uint4v{0u, 0u, 0u, 0u};
          r.dx_sgn[q] = s_sgn[e];
        }
      } else if (MODE == MODE_DX) {
        const int kraw = k0 + 8 * (pt & 7);
        const int kabs = RAGK ? min(kraw, k_end - 8) : kraw;
        const int kt = tile_div(kabs, a.Z2, p.z2_shift) * TN + step_shift(step), kin = tile_mod(kabs, a.Z2, p.z2_shift);
        const float keep = (!RAGK || kraw < k_end) ? 1.f : 0.f;
#pragma unroll
        for (int q = 0; q < Ctx::DX_LOADS; ++q) {
          const int e = kt + c.dx_ent[q];
          const float* src = p.M + s_off[e] + c.dx_rowoff[q] + kin;
          const f4u m0v = *reinterpret_cast<const f4u*>(src);
          const f4u m1v = *reinterpret_cast<const f4u*>(src + 4);
          r.dx_reg[2 * q] = floatx4{keep * m0v.v[0], keep * m0v.v[1], keep * m0v.v[2], keep * m0v.v[3]};
          r.dx_reg[2 * q + 1] = floatx4{keep * m1v.v[0], keep * m1v.v[1], keep * m1v.v[2], keep * m1v.v[3]};
          r.dx_sgn[q] = s_sgn[e];
        }
      }
      __builtin_amdgcn_sched_barrier(0);
    };

    auto store_lds = [&](RegSet<MODE, BM, BN, SHADOW>& r, int step) {
      char* Bt = b_stage(step);
      if (MODE == MODE_FWD && SHADOW) {
        // flipping the sign bit of a bf16 equals rounding the negated fp32 value
        const uint32_t flip = r.fw_sgn < 0.f ? 0x80008000u : 0u;
        const int kb4 = pt / Ctx::FS_NG;            // k = 4*kb4 .. +3: half a 16-byte chunk per column
#pragma unroll
        for (int cc = 0; cc < 8; ++cc) {
          if (Ctx::FS_NG < 16 && kb4 >= 16) break;
          const uint32_t sel = (cc & 1) ? 0x07060302u : 0x05040100u;
          const uint2v o = {__builtin_amdgcn_perm(r.fs_reg[1][cc >> 1], r.fs_reg[0][cc >> 1], sel) ^ flip,
                            __builtin_amdgcn_perm(r.fs_reg[3][cc >> 1], r.fs_reg[2][cc >> 1], sel) ^ flip};
          *reinterpret_cast<uint2v*>(Bt + lds_off(8 * (pt % Ctx::FS_NG) + cc, kb4 >> 1) + 8 * (kb4 & 1)) = o;
        }
      } else if (MODE == MODE_FWD) {
        const float sg = r.fw_sgn;
#pragma unroll
        for (int b = 0; b < Ctx::FW_BLK; ++b)
#pragma unroll
          for (int cc = 0; cc < 4; ++cc) {
            uint4v o;
#pragma unroll
            for (int pr = 0; pr < 4; ++pr)
              o[pr] = pack_bf16x2(r.fw_reg[b * 8 + 2 * pr][cc] * sg, r.fw_reg[b * 8 + 2 * pr + 1][cc] * sg);
            *reinterpret_cast<uint4v*>(Bt + lds_off(4 * (pt % Ctx::FW_NG) + cc, pt / Ctx::FW_NG + Ctx::FW_KBS * b)) = o;
          }
      } else if (MODE == MODE_DX && SHADOW) {
#pragma unroll
        for (int q = 0; q < Ctx::DX_LOADS; ++q) {
          const uint32_t flip = r.dx_sgn[q] < 0.f ? 0x80008000u : 0u;
          const uint4v v = r.ds_reg[q];
          *reinterpret_cast<uint4v*>(Bt + lds_off((pt >> 3) + 32 * q, pt & 7)) = uint4v{v[0] ^ flip, v[1] ^ flip, v[2] ^ flip, v[3] ^ flip};
        }
      } else if (MODE == MODE_DX) {
#pragma unroll
        for (int q = 0; q < Ctx::DX_LOADS; ++q) {
          const floatx4 u = r.dx_reg[2 * q], v = r.dx_reg[2 * q + 1];
          const float sg = r.dx_sgn[q];
          uint4v o = {pack_bf16x2(u[0] * sg, u[1] * sg), pack_bf16x2(u[2] * sg, u[3] * sg),
                      pack_bf16x2(v[0] * sg, v[1] * sg), pack_bf16x2(v[2] * sg, v[3] * sg)};
          *reinterpret_cast<uint4v*>(Bt + lds_off((pt >> 3) + 32 * q, pt & 7)) = o;
        }
      }
    };

    // Barrier s publishes step s: its weight tile in B stage (s & 1), written through registers
    // between barriers s-1 and s (the consumers finished reading that stage, step s-2, before
    // barrier s-1), and -- forward / dX -- its activation tile in A stage (s % 3), whose
    // direct-to-LDS loads were issued one iteration earlier (after barrier s-2, when the consumers
    // had finished step s-3) and are waited for just before barrier s.
    // Register loads run NSETS steps ahead of their use (one register set per step in flight).
    // The loop bodies are branch-free (a step index past the end is clamped and its data never
    // stored) so that the in-order wait counts can leave the newer loads in flight.  The waves that
    // have direct-to-LDS loads in flight use raw s_barrier instructions behind explicit s_waitcnt
    // values: the compiler's fence would drain every one of those loads.
    // fp32 weight tiles take twice the registers; sixteen waves leave 128 registers per lane
    constexpr int NSETS = (MODE != MODE_DM && !SHADOW) ? 2 : (NC == 8 ? 3 : 4);
    if constexpr (MODE == MODE_DM) {
      // Each role has its own loop, so that only its own transposing register sets exist.
      auto dm_loop = [&](auto* loader_type, const uint16_t* src, int64_t ld, int col, bool is_a) {
        using TL = typename std::remove_pointer<decltype(loader_type)>::type;
        TL rs[NSETS];
        const int64_t plane = is_a ? p.a_plane : p.b_plane;
        auto fetch = [&](TL& r, int step) {
          const uint16_t* from = X3 ? src + (is_a ? step_asel(step) : step_bsel(step)) * plane : src;
          r.load(from, ld, step_k0(step), I - 1, col, pt >> TL::KB_SHIFT);
        };
        auto stage = [&](TL& r, int step) {
          r.store(is_a ? a_stage(step) : b_stage(step), step_k0(step), k_end, pt & TL::COL_MASK, pt >> TL::KB_SHIFT);
        };
        const int last = nsteps - 1;
        if (nsteps > 0) {
#pragma unroll
          for (int j = 0; j < NSETS; ++j) fetch(rs[j], min(j, last));
        }
        int s = 0;
        for (; s + NSETS <= nsteps; s += NSETS) {
#pragma unroll
          for (int j = 0; j < NSETS; ++j) {
            stage(rs[j], s + j);
            fetch(rs[j], min(s + j + NSETS, last));
            __syncthreads();                             // barrier s + j
          }
        }
#pragma unroll
        for (int j = 0; j < NSETS - 1; ++j) {
          if (s + j < nsteps) {
            stage(rs[j], s + j);
            __syncthreads();
          }
        }
      };
      if (a_role) dm_loop((TLoad<BM>*)nullptr, p.A, p.lda, c.ta_col, true);
      else dm_loop((TLoad<BN>*)nullptr, p.B, p.ldb, c.tb_col, false);
      return;
    }
    if (a_producer) {
      // iteration s: fetch A(s+1), then wait until A(s) has landed (only A(s+1) is younger)
      if (nsteps > 0) dma_issue(0);
      __builtin_amdgcn_s_barrier();                      // the other waves' barrier behind the tile table
      for (int s = 0; s < nsteps; ++s) {
        dma_issue(s + 1);
        __builtin_amdgcn_s_waitcnt(vmcnt_only(Ctx::A_LOADS));
        __builtin_amdgcn_s_barrier();                    // barrier s
      }
      // Nothing may still be on its way to LDS when the consumers start to reuse the stages for
      // the epilogue (and when the waves end); the barrier pairs with the consumers' one below.
      __builtin_amdgcn_s_waitcnt(vmcnt_only(0));
      __builtin_amdgcn_s_barrier();
      return;
    }
    if constexpr (ELEM) {
      // the same two-deep pipeline as below with the gathered registers
      ElemRegs er[2];
      const int lastE = nsteps - 1;
      if (nsteps > 0) {
        elem_load(er[0], 0);
        elem_load(er[1], min(1, lastE));
      }
      int sE = 0;
      for (; sE + 2 <= nsteps; sE += 2) {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
          elem_store(er[j], sE + j);
          elem_load(er[j], min(sE + j + 2, lastE));
          __syncthreads();                               // barrier sE + j
        }
      }
      if (sE < nsteps) {
        elem_store(er[0], sE);
        __syncthreads();
      }
      __syncthreads();                                   // pairs with the consumers' barrier before the epilogue
      return;
    }
    RegSet<MODE, BM, BN, SHADOW> rs[NSETS];
    const int last = nsteps - 1;
    if (nsteps > 0) {
#pragma unroll
      for (int j = 0; j < NSETS; ++j) load_global(rs[j], min(j, last));
    }
    int s = 0;
    for (; s + NSETS <= nsteps; s += NSETS) {
#pragma unroll
      for (int j = 0; j < NSETS; ++j) {
        store_lds(rs[j], s + j);
        load_global(rs[j], min(s + j + NSETS, last));
        __syncthreads();                                 // barrier s + j
      }
    }
#pragma unroll
    for (int j = 0; j < NSETS - 1; ++j) {                // remaining steps (fewer than NSETS)
      if (s + j < nsteps) {
        store_lds(rs[j], s + j);
        __syncthreads();
      }
    }
    if constexpr (ADMA) __syncthreads();                 // pairs with the consumers' barrier before the epilogue
    return;
  }

  // ============================================================================= consumer waves
  const int wm = wave / WGN, wn = wave % WGN;
  floatx16 acc[MI][NI];
#pragma unroll
  for (int i = 0; i < MI; ++i)
#pragma unroll
    for (int j = 0; j < NI; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // Fragment addresses.  Row r0 + 32*i + (lane & 31), 16-byte chunk 2*ks + (lane >> 5): the swizzle
  // term (row ^ row >> 3) & 7 only depends on the lane and on the parity of i (32 rows flip bit 2 of
  // row >> 3, 64 rows change nothing), and 2*ks enters the chunk index by XOR -- so one offset per
  // lane and parity serves every fragment as (offset ^ ks << 5) + 8192 * (i >> 1), and no table of
  // precomputed addresses competes with the accumulators for registers.
  uint32_t a_lane[2] = {(uint32_t)lds_off(wm * WTM + (lane & 31), lane >> 5),
                        (uint32_t)lds_off(wm * WTM + 32 + (lane & 31), lane >> 5)};
  uint32_t b_lane[2] = {(uint32_t)lds_off(wn * WTN + (lane & 31), lane >> 5),
                        (uint32_t)lds_off(wn * WTN + 32 + (lane & 31), lane >> 5)};
  auto afrag = [&](const char* At, int i, int ks) {
    return *reinterpret_cast<const bf16x8*>(At + ((a_lane[i & 1] ^ (uint32_t)(ks << 5)) + (uint32_t)((i >> 1) * 8192)));
  };
  auto bfrag = [&](const char* Bt, int j, int ks) {
    return *reinterpret_cast<const bf16x8*>(Bt + ((b_lane[j & 1] ^ (uint32_t)(ks << 5)) + (uint32_t)((j >> 1) * 8192)));
  };
  // FWD / DX issue the MFMA with the operands swapped (weight fragment first), so that a lane ends
  // up with 4 consecutive output columns of one output row -- what the coalesced epilogue needs.
  // Fragments of sub-step ks+1 are requested before the MFMAs of sub-step ks are issued.
  // The loop is rotated by a quarter step: barrier s+1 sits before the last sub-step of step s, when
  // every fragment of step s is already in registers, and the first fragments of step s+1 are
  // requested right behind it -- the MFMAs of two sub-steps are queued while a wave waits at the
  // barrier, and no LDS latency is exposed after it.  (Reading step s is over before barrier s+1, so
  // the producers' rule "a stage may be refilled once the barrier after its step is passed" holds.)
  bf16x8 af[2][MI], bfr[2][NI];
  auto fetch = [&](int step, int ks, int buf) {
    const char* At = a_stage(step);
    const char* Bt = b_stage(step);
#pragma unroll
    for (int i = 0; i < MI; ++i) af[buf][i] = afrag(At, i, ks);
#pragma unroll
    for (int j = 0; j < NI; ++j) bfr[buf][j] = bfrag(Bt, j, ks);
  };
  // A block of a strip that is not its last cannot be staged through the operand stages (they are
  // busy with the next block), and storing the accumulators as they lie -- 8 bytes per lane, 32 rows
  // per instruction -- costs as much as a workgroup's whole fixed cost (measured: 4 us per block on
  // the BERT-FFN forward).  A strip's tile table is short (the host sees to it), so the unused tail of
  // the offset table serves as a small staging area: each wave passes its tile through its own
  // 8 rows x 128 bytes, eight rows at a time, and stores them 16 bytes per lane, row-contiguous.
  // The same wave writes and reads: LDS operations of one wave complete in order.
  constexpr int kStripStageRows = 8;
  static_assert(WTN != 64 || kStripTable * 8 + NC * kStripStageRows * EPI_STRIDE <= kMaxTable * 8,
                "a strip's tile table and its staging rows share the offset table's space");
  [[maybe_unused]] auto store_block_staged = [&](int t) {
    if constexpr (WTN == 64) {
      char* ebuf = reinterpret_cast<char*>(s_off) + kMaxTable * 8 - (NC - wave) * (kStripStageRows * EPI_STRIDE);
      const int cb = n0 + t * BN + wn * WTN;
      const int lr = lane & 31;
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int r8 = 0; r8 < 32 / kStripStageRows; ++r8) {
          if ((lr >> 3) == r8) {
#pragma unroll
            for (int j = 0; j < NI; ++j)
#pragma unroll
              for (int q = 0; q < 4; ++q) {
                const uint2v w = {pack_bf16x2(a.lambda * acc[i][j][4 * q], a.lambda * acc[i][j][4 * q + 1]),
                                  pack_bf16x2(a.lambda * acc[i][j][4 * q + 2], a.lambda * acc[i][j][4 * q + 3])};
                *reinterpret_cast<uint2v*>(ebuf + (lr & 7) * EPI_STRIDE + (j * 32 + 8 * q + 4 * (lane >> 5)) * 2) = w;
              }
          }
          const uint4v v = *reinterpret_cast<const uint4v*>(ebuf + (lane >> 3) * EPI_STRIDE + (lane & 7) * 16);
          const int row = m0 + wm * WTM + i * 32 + r8 * kStripStageRows + (lane >> 3);
          if (row < Mdim)
            __builtin_nontemporal_store(v, reinterpret_cast<uint4v*>(p.C + (int64_t)row * p.ldc + cb + (lane & 7) * 8));
        }
    }
  };
  int blk = 0, k_in_blk = 0;                             // strip: current block and steps done in it
  if (nsteps > 0) {
    __syncthreads();                                     // barrier 0: stages hold step 0
    fetch(0, 0, 0);
  }
  for (int s = 0; s < nsteps; ++s) {
    // (opaque to the optimiser, so that the per-fragment addresses are formed in the loop from these
    // four values instead of being kept in two dozen registers across it)
    asm volatile("" : "+v"(a_lane[0]), "+v"(a_lane[1]), "+v"(b_lane[0]), "+v"(b_lane[1]));
#pragma unroll
    for (int ks = 0; ks < BK / 16; ++ks) {
      if (ks + 1 < BK / 16) {
        fetch(s, ks + 1, (ks + 1) & 1);
      } else if (s + 1 < nsteps) {
        __syncthreads();                                 // barrier s+1: stages hold step s+1
        fetch(s + 1, 0, 0);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < MI; ++i)
#pragma unroll
        for (int j = 0; j < NI; ++j) {
          if (MODE == MODE_DM)
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[ks & 1][i], bfr[ks & 1][j], acc[i][j], 0, 0, 0);
          else
            acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(bfr[ks & 1][j], af[ks & 1][i], acc[i][j], 0, 0, 0);
        }
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (MODE != MODE_DM && !X3 && !ELEM && WTN == 64) {
      if (NTL > 1 && ++k_in_blk == nsteps_k && s + 1 < nsteps) {
        // a block of the strip is complete and another follows (its first fragments are already in
        // registers): store it and start over
        store_block_staged(blk);
        ++blk;
        k_in_blk = 0;
#pragma unroll
        for (int i = 0; i < MI; ++i)
#pragma unroll
          for (int j = 0; j < NI; ++j)
#pragma unroll
            for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;
      }
    }
  }
  // ---- epilogue (consumer waves only): the last (or only) block of the strip
  const int n0e = n0 + (NTL - 1) * BN;
  if (MODE != MODE_DM) {
    __syncthreads();   // every wave is done with the operand stages: they become the staging buffers
    // acc[i][j][e]: output row = i*32 + (lane & 31), column = j*32 + 8*(e/4) + 4*(lane >> 5) + e%4.
    // Each wave stages one 32-row block at a time in its own LDS buffer and writes it out 16 bytes
    // per lane, row-contiguous.
    if (X3 || p.G != nullptr) {
      // fp32 out: the result itself (X3), or, with a split contraction, this workgroup's partial
      // tile, which goes to its part of the workspace
      constexpr int ES = WTN * 4 + 16;          // bytes per staged row
      constexpr int CPR = WTN / 4, RPI = 64 / CPR;
      static_assert(NC * 32 * ES <= TILES_BYTES, "fp32 epilogue staging must fit in the operand stages");
      char* ebuf = smem + wave * (32 * ES);
      float* part = p.G ? p.G + (int64_t)bz * Mdim * Ndim : p.C32;
      const int64_t ldp = p.G ? (int64_t)Ndim : p.ldc;
#pragma unroll
      for (int i = 0; i < MI; ++i) {
#pragma unroll
        for (int j = 0; j < NI; ++j)
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            float4v w = {a.lambda * acc[i][j][4 * q], a.lambda * acc[i][j][4 * q + 1],
                         a.lambda * acc[i][j][4 * q + 2], a.lambda * acc[i][j][4 * q + 3]};
            *reinterpret_cast<float4v*>(ebuf + (lane & 31) * ES + (j * 32 + 8 * q + 4 * (lane >> 5)) * 4) = w;
          }
#pragma unroll
        for (int it = 0; it < (32 + RPI - 1) / RPI; ++it) {
          const int r = it * RPI + lane / CPR, cc = lane % CPR;
          if ((64 % CPR != 0) && (lane / CPR >= RPI || r >= 32)) continue;   // (only when CPR does not divide 64)
          const float4v v = *reinterpret_cast<const float4v*>(ebuf + r * ES + cc * 16);
          const int row = m0 + wm * WTM + i * 32 + r, col = n0e + wn * WTN + cc * 4;
          if (row < Mdim && col < Ndim) {
            // partial tiles are read again by the finishing kernel; a final result is not
            if (p.G) *reinterpret_cast<float4v*>(part + row * ldp + col) = v;
            else __builtin_nontemporal_store(v, reinterpret_cast<float4v*>(part + row * ldp + col));
          }
        }
      }
      return;
    }
    char* ebuf = smem + wave * (32 * EPI_STRIDE);
    constexpr int CPR = WTN / 8;              // 16-byte chunks per row of the wave tile
    constexpr int RPI = 64 / CPR;             // rows per store instruction
#pragma unroll
    for (int i = 0; i < MI; ++i) {
#pragma unroll
      for (int j = 0; j < NI; ++j)
#pragma unroll
        for (int q = 0; q < 4; ++q) {
          uint2v w = {pack_bf16x2(a.lambda * acc[i][j][4 * q], a.lambda * acc[i][j][4 * q + 1]),
                      pack_bf16x2(a.lambda * acc[i][j][4 * q + 2], a.lambda * acc[i][j][4 * q + 3])};
          *reinterpret_cast<uint2v*>(ebuf + (lane & 31) * EPI_STRIDE + (j * 32 + 8 * q + 4 * (lane >> 5)) * 2) = w;
        }
      // same wave wrote and reads: LDS operations of one wave complete in order
#pragma unroll
      for (int it = 0; it < (32 + RPI - 1) / RPI; ++it) {
        const int r = it * RPI + lane / CPR, cc = lane % CPR;
        if ((64 % CPR != 0) && (lane / CPR >= RPI || r >= 32)) continue;     // (only when CPR does not divide 64)
        const uint4v v = *reinterpret_cast<const uint4v*>(ebuf + r * EPI_STRIDE + cc * 16);
        const int row = m0 + wm * WTM + i * 32 + r, col = n0e + wn * WTN + cc * 8;
        if (row < Mdim && col < Ndim) __builtin_nontemporal_store(v, reinterpret_cast<uint4v*>(p.C + (int64_t)row * p.ldc + col));
      }
    }
  } else {
    // acc[i][j][e]: row (h) = 8*(e/4) + 4*(lane >> 5) + e%4, column (o) = lane & 31 inside the block
    const int lr = 4 * (lane >> 5), lc = lane & 31;
    if constexpr (ELEM) {
      if (p.G == nullptr) {
        // One hash per accumulator element: the column's terms of the two hashes once per 32 x 32
        // block, the row's per element.  (Indices are compile-time constants throughout, so the
        // accumulators stay in registers however large this gets.)
        const uint32_t P32 = (uint32_t)a.hash.P.d;
        const uint64_t L = bmod(a.layer, a.hash.P);
        static_for<MI * NI>([&](auto IJ) {
          constexpr int i = decltype(IJ)::value / NI, j = decltype(IJ)::value % NI;
          const int hb = m0 + wm * WTM + i * 32, ob = n0 + wn * WTN + j * 32;
          const int o = ob + lc;
          const int oc = min(o, (int)a.O - 1);
          const uint64_t y = (uint64_t)(oc / a.Z2);
          const int oin = oc % a.Z2;
          const uint32_t col_u = (uint32_t)bmod(bmod(a.hash.a0 * L, a.hash.P) + bmod(a.hash.a2 * y, a.hash.P) + a.hash.a3, a.hash.P);
          const uint32_t col_s = (uint32_t)bmod(bmod(a.hash.s0 * L, a.hash.P) +
                                                bmod(a.hash.s2 * (a.hash.use_sign == 2 ? (uint64_t)oc : y), a.hash.P) + a.hash.s3,
                                                a.hash.P);
          static_for<16>([&](auto E) {
            constexpr int e = decltype(E)::value;
            const int h = hb + 8 * (e >> 2) + lr + (e & 3);
            const int hc = min(h, (int)a.H - 1);
            const uint64_t x = (uint64_t)(hc / a.Z1);
            const int hin = hc % a.Z1;
            const uint32_t u = addmod32(col_u, (uint32_t)bmod(a.hash.a1 * x, a.hash.P), P32);
            float sc = a.lambda;
            if (a.hash.use_sign != 0) {
              const uint64_t key = a.hash.use_sign == 2 ? (uint64_t)hc : x;
              if (addmod32(col_s, (uint32_t)bmod(a.hash.s1 * key, a.hash.P), P32) & 1u) sc = -sc;
            }
            float* d = p.dM + (int64_t)((uint64_t)a.hash.align * mod_slots32(a.hash, u)) + (int64_t)a.Z2 * hin + oin;
            if (h < (int)a.H && o < (int)a.O) unsafeAtomicAdd(d, sc * acc[i][j][e]);
          });
        });
        return;
      }
    }
#pragma unroll
    for (int i = 0; i < MI; ++i)
#pragma unroll
      for (int j = 0; j < NI; ++j) {
        const int hb = m0 + wm * WTM + i * 32;      // block origin
        const int ob = n0 + wn * WTN + j * 32;
        if (hb >= (int)a.H || ob >= (int)a.O) continue;
        if (p.G) {
          float* g = p.G + ((int64_t)bz * a.H + hb) * a.O + ob + lc;
#pragma unroll
          for (int e = 0; e < 16; ++e) {
            const int r = 8 * (e >> 2) + lr + (e & 3);
            if (hb + r < (int)a.H && ob + lc < (int)a.O) g[(int64_t)r * a.O] = acc[i][j][e];
          }
        } else {
          // a lane's four consecutive rows (e % 4) share a hash tile (Z1 % 4 == 0); its column has
          // its own tile column: one table lookup per group of four values
          const int o = ob + lc, yl = tile_div(o, a.Z2, p.z2_shift) - tile_div(n0, a.Z2, p.z2_shift), oin = tile_mod(o, a.Z2, p.z2_shift);
#pragma unroll
          for (int q = 0; q < 4; ++q) {
            const int h = hb + 8 * q + lr;
            const int ent = (tile_div(h, a.Z1, p.z1_shift) - tile_div(m0, a.Z1, p.z1_shift)) * TN + yl;
            const float sc = a.lambda * s_sgn[ent];
            float* d = p.dM + s_off[ent] + (int64_t)a.Z2 * tile_mod(h, a.Z1, p.z1_shift) + oin;
#pragma unroll
            for (int r = 0; r < 4; ++r)
              if (h + r < (int)a.H && o < (int)a.O) unsafeAtomicAdd(d + (int64_t)r * a.Z2, sc * acc[i][j][4 * q + r]);
          }
        }
      }
  }
}

template <int MODE, int BM, int BN>
constexpr int smem_bytes() { return ((MODE != MODE_DM ? 3 : 2) * BM + 2 * BN) * 128 + kMaxTable * 12; }

template <int MODE, int BM, int BN, int WGM, int WGN, bool SHADOW, bool X3 = false, bool RAGK = false, bool ELEM = false>
roast_status launch(KernArgs p, dim3 blocks, hipStream_t s) {
  const int64_t total = (int64_t)blocks.x * blocks.y * blocks.z;
  if (total > (1ll << 30)) return ROAST_ERR_UNSUPPORTED;
  p.nbx = (int)blocks.x; p.nby = (int)blocks.y; p.nbz = (int)blocks.z;
  auto log2_or_minus1 = [](int z) { int sh = 0; while ((1ll << sh) < (long long)z) ++sh; return (1ll << sh) == (long long)z ? sh : -1; };
  p.z1_shift = log2_or_minus1(p.a.Z1);
  p.z2_shift = log2_or_minus1(p.a.Z2);
  const dim3 grid((unsigned)((total + 7) / 8 * 8));
  constexpr int smem = smem_bytes<MODE, BM, BN>();
  static_assert(smem <= 160 * 1024, "LDS budget");
  static std::atomic<bool> configured{false};   // per instantiation and process; a race between host threads only repeats the call
  if (!configured.load(std::memory_order_acquire)) {
    if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_roast_mfma<MODE, BM, BN, WGM, WGN, SHADOW, X3, RAGK, ELEM>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, smem) != hipSuccess)
      return ROAST_ERR_HIP;
    configured.store(true, std::memory_order_release);
  }
  hipLaunchKernelGGL((k_roast_mfma<MODE, BM, BN, WGM, WGN, SHADOW, X3, RAGK, ELEM>), grid, dim3((WGM * WGN + 8) * 64),
                     smem, s, p);
  return hip_status(hipGetLastError());
}

// out[i] = bf16(M[i]) and out[stride + i] = bf16(M[i + 1]), zero beyond the end of M
__global__ __launch_bounds__(256) void k_shadow_bf16(const float* __restrict__ M, int64_t n, int64_t stride,
                                                     uint16_t* __restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= stride) return;
  const uint16_t cur = i < n ? __builtin_bit_cast(uint16_t, (__bf16)M[i]) : (uint16_t)0;
  const uint16_t nxt = i + 1 < n ? __builtin_bit_cast(uint16_t, (__bf16)M[i + 1]) : (uint16_t)0;
  out[i] = cur;
  out[stride + i] = nxt;
}

// C[r][c] = bf16(sum over the parts, in order, of G[part][r][c]); eight columns per thread
__global__ __launch_bounds__(256) void k_split_finish(const float* __restrict__ G, int parts, int64_t rows,
                                                      int64_t cols, uint16_t* __restrict__ C, int64_t ldc) {
  const int64_t cpr = cols / 8;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= rows * cpr) return;
  const int64_t r = t / cpr, c = (t % cpr) * 8;
  float4v s0 = {0.f, 0.f, 0.f, 0.f}, s1 = s0;
  for (int q = 0; q < parts; ++q) {
    const float4v* g = reinterpret_cast<const float4v*>(G + ((int64_t)q * rows + r) * cols + c);
    s0 += g[0];
    s1 += g[1];
  }
  const uint4v v = {pack_bf16x2(s0[0], s0[1]), pack_bf16x2(s0[2], s0[3]), pack_bf16x2(s1[0], s1[1]),
                    pack_bf16x2(s1[2], s1[3])};
  *reinterpret_cast<uint4v*>(C + r * ldc + c) = v;
}

// fp32 -> three bfloat16 values with x == hi + mid + lo exactly: each plane takes the leading 8
// significand bits of what is left (truncation, so the partial sums hi, hi + mid, ... grow
// monotonically towards x and cannot overflow).  Each residual is exact in fp32.  Below 2^-110 the
// residuals become subnormal and lose their low bits (absolute error below 2^-133).  Inf / NaN stay
// in the first plane (their products with the zero planes of the other operand are NaN).
__device__ inline void split3(float x, uint16_t* hi, uint16_t* mid, uint16_t* lo) {
  const uint32_t bits = __builtin_bit_cast(uint32_t, x);
  if ((bits & 0x7f800000u) == 0x7f800000u) {
    *hi = (uint16_t)((bits >> 16) | ((bits & 0xffffu) ? 0x40u : 0u));   // keep a NaN a NaN
    *mid = *lo = 0;
    return;
  }
  const uint32_t h = bits & 0xffff0000u;
  const float r1 = x - __builtin_bit_cast(float, h);
  const uint32_t m = __builtin_bit_cast(uint32_t, r1) & 0xffff0000u;
  const float r2 = r1 - __builtin_bit_cast(float, m);
  *hi = (uint16_t)(h >> 16);
  *mid = (uint16_t)(m >> 16);
  *lo = (uint16_t)(__builtin_bit_cast(uint32_t, r2) >> 16);
}

// planes[s][r * ldo + c] = plane s of src[r * ld + c]; VEC consecutive columns per thread
// (VEC = 4: 16-byte loads, 8-byte stores; needs cols % 4 == 0, ld % 4 == 0 and a 16-byte aligned src)
template <int VEC>
__global__ __launch_bounds__(256) void k_split3_rows(const float* __restrict__ src, int64_t rows, int64_t cols,
                                                     int64_t ld, uint16_t* __restrict__ out, int64_t ldo,
                                                     int64_t plane) {
  const int64_t cpr = cols / VEC;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= rows * cpr) return;
  const int64_t r = t / cpr, c = (t - r * cpr) * VEC;
  uint16_t h[VEC], m[VEC], l[VEC];
  if constexpr (VEC == 4) {
    const float4v v = __builtin_nontemporal_load(reinterpret_cast<const float4v*>(src + r * ld + c));
#pragma unroll
    for (int i = 0; i < 4; ++i) split3(v[i], &h[i], &m[i], &l[i]);
  } else {
    split3(src[r * ld + c], &h[0], &m[0], &l[0]);
  }
  uint16_t* o = out + r * ldo + c;
  if constexpr (VEC == 4) {
    *reinterpret_cast<uint2v*>(o) = uint2v{(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
    *reinterpret_cast<uint2v*>(o + plane) = uint2v{(uint32_t)m[0] | ((uint32_t)m[1] << 16), (uint32_t)m[2] | ((uint32_t)m[3] << 16)};
    *reinterpret_cast<uint2v*>(o + 2 * plane) = uint2v{(uint32_t)l[0] | ((uint32_t)l[1] << 16), (uint32_t)l[2] | ((uint32_t)l[3] << 16)};
  } else {
    o[0] = h[0];
    o[plane] = m[0];
    o[2 * plane] = l[0];
  }
}

// Three shadows of M, one per plane, each in the two-copy layout of k_shadow_bf16:
// out[s * 2 * stride + i] = plane s of M[i], out[s * 2 * stride + stride + i] = plane s of M[i + 1]
__global__ __launch_bounds__(256) void k_shadow3(const float* __restrict__ M, int64_t n, int64_t stride,
                                                 uint16_t* __restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i >= stride) return;
  uint16_t c[3] = {0, 0, 0}, x[3] = {0, 0, 0};
  if (i < n) split3(M[i], &c[0], &c[1], &c[2]);
  if (i + 1 < n) split3(M[i + 1], &x[0], &x[1], &x[2]);
#pragma unroll
  for (int s = 0; s < 3; ++s) {
    out[(int64_t)s * 2 * stride + i] = c[s];
    out[(int64_t)s * 2 * stride + stride + i] = x[s];
  }
}

// fp32 result of a split contraction: C[r][c] = sum over the parts, in order, of G[part][r][c]
__global__ __launch_bounds__(256) void k_split_finish_f32(const float* __restrict__ G, int parts, int64_t rows,
                                                          int64_t cols, float* __restrict__ C, int64_t ldc) {
  const int64_t cpr = cols / 4;
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (t >= rows * cpr) return;
  const int64_t r = t / cpr, c = (t % cpr) * 4;
  float4v sum = {0.f, 0.f, 0.f, 0.f};
  for (int q = 0; q < parts; ++q) sum += *reinterpret_cast<const float4v*>(G + ((int64_t)q * rows + r) * cols + c);
  *reinterpret_cast<float4v*>(C + r * ldc + c) = sum;
}

inline int64_t shadow_stride_of(int64_t m_size) { return (m_size + 1 + 63) / 64 * 64; }
inline bool aligned16(const void* p) { return ((uintptr_t)p & 15) == 0; }
inline int64_t cdiv(int64_t a, int64_t b) { return (a + b - 1) / b; }
// True when blocks of kBNarrow columns fill the 256 CUs in fewer or shorter rounds than blocks of
// kBN columns do (rb row blocks, n output columns): 8192 x 768 outputs are 192 blocks of 128 columns
// but exactly 256 of 96.
inline bool narrow_pays(int64_t rb, int64_t n) {
  return cdiv(rb * cdiv(n, kBNarrow), 256) * kBNarrow < cdiv(rb * cdiv(n, kBN), 256) * kBN;
}

// Column blocks per workgroup strip for a forward / dX launch with rb row blocks, n output columns,
// hash tiles of z columns, `steps` contraction steps per block and tiles_k hash tiles along the
// contraction.  Model (microseconds, fitted to the BERT-FFN and BERT-QKV shapes): a step takes 1.2,
// a workgroup 3.3 of fixed cost (launch, tile table, first loads, the staged epilogue and its drain),
// a further block of a strip 0.9 (its stores through the small staging area); workgroups beyond 256
// queue, a last partial round counting half.  Strips need whole blocks of whole hash tiles
// (n % (kBN * t) == 0, kBN % z == 0) and a tile table short enough to leave the staging rows free;
// the candidate with the smallest modelled time wins, so strips form where short blocks would
// otherwise queue for the CUs (8192 x 768 -> 3072: three rounds of 12-step blocks become one round
// of 36-step strips, 58 -> 53 us) and not where they would leave CUs idle.
inline int pick_ntile(int64_t rb, int64_t n, int64_t z, int64_t steps, int64_t tiles_k) {
  if (z <= 0 || kBN % z != 0) return 1;
  int best = 1;
  double best_cost = 0.0;
  for (int t = 1; t <= 4; ++t) {
    if (n % ((int64_t)kBN * t) != 0 || tiles_k * ((int64_t)kBN * t / z) > (t == 1 ? kMaxTable : kStripTable)) continue;
    const double wgs = (double)(rb * (n / ((int64_t)kBN * t)));
    const double rounds = wgs <= 256.0 ? 1.0 : 0.5 * ((double)cdiv((int64_t)wgs, 256) + wgs / 256.0);
    const double cost = rounds * ((double)(t * steps) * 1.2 + 3.3 + 0.9 * (t - 1));
    if (t == 1 || cost < best_cost) { best_cost = cost; best = t; }
  }
  return best;
}

}  // namespace


int64_t shadow_stride(int64_t m_size) { return shadow_stride_of(m_size); }

roast_status shadow_bf16_launch(const float* M, int64_t m_size, void* shadow, hipStream_t s) {
  const int64_t stride = shadow_stride(m_size);
  const int64_t blocks = (stride + 255) / 256;
  if (blocks > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
  hipLaunchKernelGGL(k_shadow_bf16, dim3((unsigned)blocks), dim3(256), 0, s, M, m_size, stride, (uint16_t*)shadow);
  return hip_status(hipGetLastError());
}

namespace {

// Sets up a split of the contraction axis (length K) into `splits` parts of whole 64-steps.
void split_setup(KernArgs* p, dim3* grid, int64_t K, int splits, float* ws) {
  if (splits <= 1 || ws == nullptr) return;
  p->rows_per_split = (int)(cdiv(cdiv(K, splits), BK) * BK);
  p->G = ws;
  grid->z = (unsigned)cdiv(K, p->rows_per_split);
}

roast_status split_finish(const KernArgs& p, unsigned parts, int64_t rows, int64_t cols, hipStream_t s) {
  if (p.G == nullptr) return ROAST_OK;
  const int64_t blocks = cdiv(rows * (cols / (p.C32 ? 4 : 8)), 256);
  if (blocks > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
  if (p.C32)
    hipLaunchKernelGGL(k_split_finish_f32, dim3((unsigned)blocks), dim3(256), 0, s, p.G, (int)parts, rows, cols, p.C32,
                       p.ldc);
  else
    hipLaunchKernelGGL(k_split_finish, dim3((unsigned)blocks), dim3(256), 0, s, p.G, (int)parts, rows, cols, p.C, p.ldc);
  return hip_status(hipGetLastError());
}

inline size_t up256(size_t v) { return (v + 255) / 256 * 256; }
inline int64_t pad8(int64_t v) { return (v + 7) / 8 * 8; }

// planes of a rows x cols fp32 matrix: 3 x rows x pad8(cols) bfloat16
size_t planes_bytes(int64_t rows, int64_t cols) { return up256((size_t)3 * rows * pad8(cols) * 2); }
size_t shadow3_bytes(int64_t m_size) { return up256((size_t)3 * 2 * shadow_stride_of(m_size) * 2); }

roast_status split_rows(const float* src, int64_t rows, int64_t cols, int64_t ld, uint16_t* out, hipStream_t s) {
  const bool vec = cols % 4 == 0 && ld % 4 == 0 && aligned16(src);
  const int64_t blocks = cdiv(rows * (vec ? cols / 4 : cols), 256);
  if (blocks > 0x7fffffffll) return ROAST_ERR_UNSUPPORTED;
  if (vec)
    hipLaunchKernelGGL(k_split3_rows<4>, dim3((unsigned)blocks), dim3(256), 0, s, src, rows, cols, ld, out, pad8(cols),
                       rows * pad8(cols));
  else
    hipLaunchKernelGGL(k_split3_rows<1>, dim3((unsigned)blocks), dim3(256), 0, s, src, rows, cols, ld, out, pad8(cols),
                       rows * pad8(cols));
  return hip_status(hipGetLastError());
}

roast_status shadow3(const float* M, int64_t m_size, uint16_t* out, hipStream_t s) {
  const int64_t stride = shadow_stride_of(m_size);
  hipLaunchKernelGGL(k_shadow3, dim3((unsigned)cdiv(stride, 256)), dim3(256), 0, s, M, m_size, stride, out);
  return hip_status(hipGetLastError());
}

// (the tile table holds one sign per tile: per-element signs, use_sign == 2, and tiles that break the
// rules below take the element-wise instantiations, one hash per virtual weight)
// The contraction runs in 64-deep steps; its length (H resp. O) only has to be a multiple of 8: the
// last step's surplus is staged as zero weights.  A load thread's block of the weight tile -- 8 rows of the contraction axis (forward), 8 consecutive elements of it (dX) --
// must lie inside one hash tile, which may be smaller than the step.
bool mfma_fwd_ok(const MMArgs& a) {
  return a.hash.use_sign != 2 && a.Z1 % 8 == 0 && a.H % 8 == 0 && a.Z2 % 4 == 0 && a.O % 8 == 0 &&
         a.nTx * (cdiv(kBN, a.Z2) + 1) <= kMaxTable;
}
bool mfma_dx_ok(const MMArgs& a) {
  return a.hash.use_sign != 2 && a.Z2 % 8 == 0 && a.O % 8 == 0 && a.H % 8 == 0 &&
         a.nTy * (cdiv(kBN, a.Z1) + 1) <= kMaxTable;
}
// element-wise staging: any tile shape and sign mode; the activations still go to LDS in 16-byte pieces
bool mfma_elem_ok(const MMArgs& a) { return a.H % 8 == 0 && a.O % 8 == 0; }

}  // namespace

// Blocks per strip of a forward / dX launch whose contraction is not split (1 wherever the launch
// takes another instantiation: element-wise, ragged contraction, narrow blocks).
int mfma_fwd_strip(const MMArgs& a, bool shadow) {
  if (!mfma_fwd_ok(a) || a.H % BK != 0) return 1;
  if (shadow && a.Z2 % 8 == 0 && narrow_pays(cdiv(a.I, kBM), a.O)) return 1;
  return pick_ntile(cdiv(a.I, kBM), a.O, a.Z2, a.H / BK, a.nTx);
}
int mfma_dx_strip(const MMArgs& a, bool shadow) {
  if (!mfma_dx_ok(a) || a.O % BK != 0) return 1;
  if (shadow && narrow_pays(cdiv(a.I, kBM), a.H)) return 1;
  return pick_ntile(cdiv(a.I, kBM), a.H, a.Z1, a.O / BK, a.nTy);
}

int mfma_fwd_splits(const MMArgs& a) {
  return (mfma_fwd_ok(a) || mfma_elem_ok(a)) ? mm_pick_splits(cdiv(a.O, kBN) * cdiv(a.I, kBM), a.H) : 1;
}
int mfma_dx_splits(const MMArgs& a) {
  return (mfma_dx_ok(a) || mfma_elem_ok(a)) ? mm_pick_splits(cdiv(a.H, kBN) * cdiv(a.I, kBM), a.O) : 1;
}

roast_status mfma_mm_fwd(const MMArgs& a, const void* X, int64_t ldx, const float* M, const void* M_bf16, void* Y,
                         int64_t ldy, float* ws, hipStream_t s) {
  const bool elem = !mfma_fwd_ok(a);
  if ((elem && !mfma_elem_ok(a)) || ldx % 8 != 0 || ldy % 8 != 0 || !aligned16(X) || !aligned16(Y))
    return ROAST_ERR_UNSUPPORTED;
  constexpr int BM = kBM, BN = kBN;
  KernArgs p{};
  p.a = a; p.A = (const uint16_t*)X; p.lda = ldx; p.M = M; p.Mb = (const uint16_t*)M_bf16;
  p.mb_stride = shadow_stride(a.m_size); p.C = (uint16_t*)Y; p.ldc = ldy;
  dim3 grid((unsigned)cdiv(a.O, BN), (unsigned)cdiv(a.I, BM), 1);
  split_setup(&p, &grid, a.H, mfma_fwd_splits(a), ws);
  // the shadow is read in 8-column pieces, which must not straddle tiles
  const bool shadow = M_bf16 && a.Z2 % 8 == 0;
  roast_status st;
  // a narrower block (256 x 96, eight 32 x 96 consumer tiles) when it fills the CUs better
  const bool narrow = !elem && shadow && a.H % BK == 0 && grid.z == 1 && narrow_pays(cdiv(a.I, BM), a.O);
  if (elem) {
    st = launch<MODE_FWD, BM, BN, 4, 2, false, false, true, true>(p, grid, s);
  } else if (narrow) {
    grid.x = (unsigned)cdiv(a.O, kBNarrow);
    st = launch<MODE_FWD, BM, kBNarrow, 8, 1, true>(p, grid, s);
  } else if (a.H % BK != 0)
    st = shadow ? launch<MODE_FWD, BM, BN, 4, 2, true, false, true>(p, grid, s)
                : launch<MODE_FWD, BM, BN, 4, 2, false, false, true>(p, grid, s);
  else {
    if (grid.z == 1) {
      p.ntile = mfma_fwd_strip(a, shadow);
      p.tile_shift = BN / a.Z2;
      grid.x = (unsigned)cdiv(a.O, (int64_t)BN * p.ntile);
    }
    st = shadow ? launch<MODE_FWD, BM, BN, 4, 2, true>(p, grid, s) : launch<MODE_FWD, BM, BN, 4, 2, false>(p, grid, s);
  }
  return st != ROAST_OK ? st : split_finish(p, grid.z, a.I, a.O, s);
}

roast_status mfma_mm_bwd_dx(const MMArgs& a, const void* dY, int64_t ldy, const float* M, const void* M_bf16,
                            void* dX, int64_t ldx, float* ws, hipStream_t s) {
  const bool elem = !mfma_dx_ok(a);
  if ((elem && !mfma_elem_ok(a)) || ldy % 8 != 0 || ldx % 8 != 0 || !aligned16(dY) || !aligned16(dX))
    return ROAST_ERR_UNSUPPORTED;
  constexpr int BM = kBM, BN = kBN;
  KernArgs p{};
  p.a = a; p.A = (const uint16_t*)dY; p.lda = ldy; p.M = M; p.Mb = (const uint16_t*)M_bf16;
  p.mb_stride = shadow_stride(a.m_size); p.C = (uint16_t*)dX; p.ldc = ldx;
  dim3 grid((unsigned)cdiv(a.H, BN), (unsigned)cdiv(a.I, BM), 1);
  split_setup(&p, &grid, a.O, mfma_dx_splits(a), ws);
  roast_status st;
  const bool narrow = !elem && M_bf16 && a.O % BK == 0 && grid.z == 1 && narrow_pays(cdiv(a.I, BM), a.H);
  if (elem) {
    st = launch<MODE_DX, BM, BN, 4, 2, false, false, true, true>(p, grid, s);
  } else if (narrow) {
    grid.x = (unsigned)cdiv(a.H, kBNarrow);
    st = launch<MODE_DX, BM, kBNarrow, 8, 1, true>(p, grid, s);
  } else if (a.O % BK != 0)
    st = M_bf16 ? launch<MODE_DX, BM, BN, 4, 2, true, false, true>(p, grid, s)
                : launch<MODE_DX, BM, BN, 4, 2, false, false, true>(p, grid, s);
  else {
    if (grid.z == 1) {
      p.ntile = mfma_dx_strip(a, M_bf16 != nullptr);
      p.tile_shift = BN / a.Z1;
      grid.x = (unsigned)cdiv(a.H, (int64_t)BN * p.ntile);
    }
    st = M_bf16 ? launch<MODE_DX, BM, BN, 4, 2, true>(p, grid, s) : launch<MODE_DX, BM, BN, 4, 2, false>(p, grid, s);
  }
  return st != ROAST_OK ? st : split_finish(p, grid.z, a.I, a.H, s);
}

// Parts of the contraction axis for the dM product with the atomic epilogue.  All workgroups of a
// launch run at once, so with equal parts they would all reach their epilogue together and the
// atomic units (0.3 T adds/s for the whole chip) would be the only thing running for the last
// quarter of the kernel.  Parts of graded length -- proportional to 1 + d*(2z/(s-1) - 1), d = 0.22,
// in whole 64-row steps -- spread the epilogues out, so that the adds of the early workgroups
// overlap the products of the late ones (measured: 94 -> 85 us on the BERT-FFN shapes).
// A function of the shape only.
static void uneven_parts(int64_t I, int splits, int* begin) {
  if (splits < 2 || splits > 16) return;     // begin[] stays zero: equal parts of rows_per_split
  constexpr double d = 0.22;
  double acc = 0.0;
  begin[0] = 0;
  for (int z = 0; z < splits; ++z) {
    acc += (1.0 + d * (2.0 * z / (splits - 1) - 1.0)) / splits;
    int64_t e = (int64_t)(acc * (double)I / BK + 0.5) * BK;
    if (z == splits - 1 || e > I) e = I;
    begin[z + 1] = (int)e;
  }
}

roast_status mfma_mm_bwd_dM(const MMArgs& a, const void* X, int64_t ldx, const void* dY, int64_t ldy, float* dM,
                            float* Gws, int splits, hipStream_t s) {
  constexpr int BM = 256, BN = 128;
  if (a.H % 8 != 0 || a.O % 8 != 0 || ldx % 8 != 0 || ldy % 8 != 0 || !aligned16(X) || !aligned16(dY) ||
      a.H < BM / 32 || a.O < BN / 32)
    return ROAST_ERR_UNSUPPORTED;
  // The tiled epilogue looks a tile up once per four accumulator rows and applies one sign per tile;
  // other tile shapes, per-element signs and tile tables that do not fit hash every element instead
  // (raw products for the deterministic reduction carry no sign and need no table either way).
  const bool elem = a.Z1 % 4 != 0 || (Gws == nullptr && a.hash.use_sign == 2) ||
                    (cdiv(BM, a.Z1) + 1) * (cdiv(BN, a.Z2) + 1) > kMaxTable;
  const int64_t tiles = cdiv(a.H, BM) * cdiv(a.O, BN);
  if (Gws == nullptr) splits = dm_pick_splits(tiles, a.I, a.H * a.O);
  if (splits < 1 || splits > 65535) return ROAST_ERR_UNSUPPORTED;
  int64_t rows = cdiv(a.I, splits);
  rows = cdiv(rows, BK) * BK;
  KernArgs p{};
  p.a = a; p.A = (const uint16_t*)X; p.lda = ldx; p.B = (const uint16_t*)dY; p.ldb = ldy; p.dM = dM; p.G = Gws;
  p.rows_per_split = (int)rows;
  if (Gws == nullptr) uneven_parts(a.I, splits, p.split_begin);
  const dim3 grid((unsigned)cdiv(a.O, BN), (unsigned)cdiv(a.H, BM), (unsigned)splits);
  return elem ? launch<MODE_DM, BM, BN, 4, 2, false, false, false, true>(p, grid, s)
              : launch<MODE_DM, BM, BN, 4, 2, false>(p, grid, s);
}

// ---- fp32 through the three-plane kernels.  Workspace layout (every part 256-byte aligned):
// forward: [planes of X][three shadows of M][partial outputs of a split contraction]
// dX     : [planes of dY][three shadows of M][partial outputs]
// dM     : [planes of X][planes of dY]
bool x3_fwd_ok(const MMArgs& a) { return mfma_fwd_ok(a) && a.Z2 % 8 == 0 && a.O % 4 == 0; }
bool x3_dx_ok(const MMArgs& a) { return mfma_dx_ok(a) && a.H % 4 == 0; }
bool x3_dm_ok(const MMArgs& a) {
  return a.hash.use_sign != 2 && a.Z1 % 4 == 0 && a.H % 8 == 0 && a.O % 8 == 0 && a.H >= kBM / 32 && a.O >= kBN / 32 &&
         (cdiv(kBM, a.Z1) + 1) * (cdiv(kBN, a.Z2) + 1) <= kMaxTable;
}
int x3_fwd_splits(const MMArgs& a) { return mm_pick_splits(cdiv(a.O, kBN) * cdiv(a.I, kBM), 6 * a.H); }
int x3_dx_splits(const MMArgs& a) { return mm_pick_splits(cdiv(a.H, kBN) * cdiv(a.I, kBM), 6 * a.O); }

size_t x3_fwd_workspace(const MMArgs& a) {
  if (!x3_fwd_ok(a)) return 0;
  const int s = x3_fwd_splits(a);
  return planes_bytes(a.I, a.H) + shadow3_bytes(a.m_size) + (s > 1 ? (size_t)s * a.I * a.O * 4 : 0);
}
size_t x3_dx_workspace(const MMArgs& a) {
  if (!x3_dx_ok(a)) return 0;
  const int s = x3_dx_splits(a);
  return planes_bytes(a.I, a.O) + shadow3_bytes(a.m_size) + (s > 1 ? (size_t)s * a.I * a.H * 4 : 0);
}
size_t x3_dm_workspace(const MMArgs& a) {
  return x3_dm_ok(a) ? planes_bytes(a.I, a.H) + planes_bytes(a.I, a.O) : 0;
}

size_t m_planes_bytes(int64_t m_size) { return shadow3_bytes(m_size); }

roast_status m_planes_launch(const float* M, int64_t m_size, void* planes, hipStream_t s) {
  return shadow3(M, m_size, (uint16_t*)planes, s);
}

roast_status x3_mm_fwd(const MMArgs& a, const float* X, int64_t ldx, const float* M, const void* M_planes, float* Y,
                       int64_t ldy, void* ws, hipStream_t s) {
  if (!x3_fwd_ok(a) || ldy % 4 != 0 || !aligned16(Y) || !aligned16(ws)) return ROAST_ERR_UNSUPPORTED;
  char* base = (char*)ws;
  uint16_t* Xp = (uint16_t*)base;
  uint16_t* Mp = (uint16_t*)(base + planes_bytes(a.I, a.H));
  float* parts = (float*)(base + planes_bytes(a.I, a.H) + shadow3_bytes(a.m_size));
  roast_status st = split_rows(X, a.I, a.H, ldx, Xp, s);
  if (st != ROAST_OK) return st;
  if (M_planes) Mp = (uint16_t*)M_planes;      // made once per update of M by the caller
  else st = shadow3(M, a.m_size, Mp, s);
  if (st != ROAST_OK) return st;
  KernArgs p{};
  p.a = a; p.A = Xp; p.lda = pad8(a.H); p.a_plane = a.I * pad8(a.H); p.M = M; p.Mb = Mp;
  p.mb_stride = shadow_stride_of(a.m_size); p.mb_plane = 2 * p.mb_stride; p.C32 = Y; p.ldc = ldy;
  dim3 grid((unsigned)cdiv(a.O, kBN), (unsigned)cdiv(a.I, kBM), 1);
  split_setup(&p, &grid, a.H, x3_fwd_splits(a), parts);
  if (grid.z == 1 && a.H % BK == 0 && narrow_pays(cdiv(a.I, kBM), a.O)) {
    grid.x = (unsigned)cdiv(a.O, kBNarrow);
    st = launch<MODE_FWD, kBM, kBNarrow, 8, 1, true, true>(p, grid, s);
  } else
    st = a.H % BK != 0 ? launch<MODE_FWD, kBM, kBN, 4, 2, true, true, true>(p, grid, s)
                       : launch<MODE_FWD, kBM, kBN, 4, 2, true, true>(p, grid, s);
  return st != ROAST_OK ? st : split_finish(p, grid.z, a.I, a.O, s);
}

roast_status x3_mm_bwd_dx(const MMArgs& a, const float* dY, int64_t ldy, const float* M, const void* M_planes,
                          float* dX, int64_t ldx, void* ws, hipStream_t s) {
  if (!x3_dx_ok(a) || ldx % 4 != 0 || !aligned16(dX) || !aligned16(ws)) return ROAST_ERR_UNSUPPORTED;
  char* base = (char*)ws;
  uint16_t* Gp = (uint16_t*)base;
  uint16_t* Mp = (uint16_t*)(base + planes_bytes(a.I, a.O));
  float* parts = (float*)(base + planes_bytes(a.I, a.O) + shadow3_bytes(a.m_size));
  roast_status st = split_rows(dY, a.I, a.O, ldy, Gp, s);
  if (st != ROAST_OK) return st;
  if (M_planes) Mp = (uint16_t*)M_planes;
  else st = shadow3(M, a.m_size, Mp, s);
  if (st != ROAST_OK) return st;
  KernArgs p{};
  p.a = a; p.A = Gp; p.lda = pad8(a.O); p.a_plane = a.I * pad8(a.O); p.M = M; p.Mb = Mp;
  p.mb_stride = shadow_stride_of(a.m_size); p.mb_plane = 2 * p.mb_stride; p.C32 = dX; p.ldc = ldx;
  dim3 grid((unsigned)cdiv(a.H, kBN), (unsigned)cdiv(a.I, kBM), 1);
  split_setup(&p, &grid, a.O, x3_dx_splits(a), parts);
  if (grid.z == 1 && a.O % BK == 0 && narrow_pays(cdiv(a.I, kBM), a.H)) {
    grid.x = (unsigned)cdiv(a.H, kBNarrow);
    st = launch<MODE_DX, kBM, kBNarrow, 8, 1, true, true>(p, grid, s);
  } else
    st = a.O % BK != 0 ? launch<MODE_DX, kBM, kBN, 4, 2, true, true, true>(p, grid, s)
                       : launch<MODE_DX, kBM, kBN, 4, 2, true, true>(p, grid, s);
  return st != ROAST_OK ? st : split_finish(p, grid.z, a.I, a.H, s);
}

roast_status x3_mm_bwd_dM(const MMArgs& a, const float* X, int64_t ldx, const float* dY, int64_t ldy, float* dM,
                          void* ws, hipStream_t s) {
  if (!x3_dm_ok(a) || !aligned16(ws)) return ROAST_ERR_UNSUPPORTED;
  char* base = (char*)ws;
  uint16_t* Xp = (uint16_t*)base;
  uint16_t* Gp = (uint16_t*)(base + planes_bytes(a.I, a.H));
  roast_status st = split_rows(X, a.I, a.H, ldx, Xp, s);
  if (st != ROAST_OK) return st;
  st = split_rows(dY, a.I, a.O, ldy, Gp, s);
  if (st != ROAST_OK) return st;
  const int64_t tiles = cdiv(a.H, kBM) * cdiv(a.O, kBN);
  const int splits = dm_pick_splits(tiles, 6 * a.I, a.H * a.O);
  int64_t rows = cdiv(a.I, splits);
  rows = cdiv(rows, BK) * BK;
  KernArgs p{};
  p.a = a; p.A = Xp; p.lda = pad8(a.H); p.a_plane = a.I * pad8(a.H);
  p.B = Gp; p.ldb = pad8(a.O); p.b_plane = a.I * pad8(a.O); p.dM = dM;
  p.rows_per_split = (int)rows;
  const unsigned parts = (unsigned)cdiv(a.I, rows);
  uneven_parts(a.I, (int)parts, p.split_begin);
  const dim3 grid((unsigned)cdiv(a.O, kBN), (unsigned)cdiv(a.H, kBM), parts);
  return launch<MODE_DM, kBM, kBN, 4, 2, false, true>(p, grid, s);
}

}  // namespace roast
