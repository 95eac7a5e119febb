/*
 * roast.h -- C-ABI of the MI355X (gfx950) ROAST hashing hot path.
 *
 * ROAST (arXiv 2207.10702) keeps every learnable parameter of a model in one small flat array M
 * and recovers weights from it block by block: a ROAST-MM layer's virtual weight matrix W (H x O)
 * is cut into Z1 x Z2 tiles, tile (x, y) is the contiguous, row-major slice of M that starts at a
 * hashed offset, times a hashed +-1 sign and a per-module scale lambda (Section 4.1, "Matrix
 * multiplication" paragraph and Algorithm 1); an embedding row is recovered the same way in 1-D
 * chunks of Z scalars (Section 4.1, "Lookup" paragraph).  W is never materialised.
 *
 * Conventions shared by every entry point
 *   - Pointers named X, Y, dY, dX, M, dM, out, dOut, rows, table_ids, ws are DEVICE pointers owned
 *     by the caller.  roast_tile_index alone takes HOST pointers.  The library never allocates,
 *     frees or keeps device memory; scratch comes in through `ws`.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls enqueue work and return; they
 *     never synchronise.  Outputs are valid once the stream reaches that point.
 *   - Matrices are row-major with a leading dimension in elements (ld >= number of columns).
 *   - M and dM are always fp32.  roast_dtype is the type of the activations X / Y / dY / dX;
 *     products are accumulated in fp32.  With ROAST_BF16 the recovered tile sign*M is rounded to
 *     bfloat16 (nearest even) when it is staged as the MFMA weight operand and lambda is applied to
 *     the fp32 accumulator.
 *   - dM is ACCUMULATED INTO (dM += ...): all layers sharing one M add into one gradient buffer
 *     (global memory sharing, Section 4.2; gradient equation of Section 4.3).  The caller zeroes it.
 *   - M is never written.  No entry point touches memory outside the extents stated below.
 *   - Errors are return codes; nothing is launched when a call returns non-zero, except
 *     ROAST_ERR_HIP which reports a launch failure from the runtime.
 *   - The HIP runtime keeps one "last error" per host thread, whoever caused it.  Every entry point
 *     that launches kernels reads -- and thereby CLEARS -- that value before it launches, so that
 *     ROAST_ERR_HIP is about this library's own launches only.  A caller that wants to see an
 *     error left behind by its own earlier HIP calls must read hipGetLastError() before it calls
 *     into this library; afterwards it is gone.
 *   - Sizes of zero rows (I == 0, N == 0) are a successful no-op.
 *   - A call only enqueues kernels on `stream`: no allocation, no synchronisation, no memset or
 *     copy.  A sequence of calls may therefore be recorded in a HIP graph, once every kernel of the
 *     sequence has run once outside the capture (a kernel's first launch in a process sets a
 *     function attribute).
 *   - Every shape within the limits below is accepted; which kernels run is a matter of speed,
 *     never of results beyond the stated tolerances.  Limits (ROAST_ERR_UNSUPPORTED beyond them):
 *     H, O, I, D < 2^31; the generic ROAST-MM kernels (any call the matrix-core kernels do not
 *     take) handle at most 65535 * 64 = 4 194 240 rows I; DETERMINISTIC roast_mm_bwd_dM at most
 *     2^17 = 131 072 tiles per layer; DETERMINISTIC lookup gradients fewer than 2^40 chunks.  The matrix-core kernels take ROAST_BF16 calls (and ROAST_F32 calls that
 *     come with a workspace, see roast_mm_fwd_ws) with 16-byte aligned pointers, leading dimensions
 *     that are multiples of 8, H and O multiples of 8, and tiles with Z1 % 8 == 0 and Z2 % 4 == 0
 *     (forward), Z2 % 8 == 0 (dX), Z1 % 4 == 0 (dM), per-block sign; the lookup kernels are fastest
 *     with Z % 4 == 0, D % Z == 0 and |M| < 2^31.  Everything else runs on generic kernels.
 */
#ifndef ROAST_H
#define ROAST_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  ROAST_OK = 0,
  ROAST_ERR_ARG = 1,         /* null pointer, negative size, ld too small, bad enum              */
  ROAST_ERR_SHAPE = 2,       /* H, O, Z1, Z2, D or Z not positive                                */
  ROAST_ERR_RANGE = 3,       /* a block does not fit (|M| < Z1*Z2 or |M| < Z), or bad hash params */
  ROAST_ERR_WORKSPACE = 4,   /* ws is null or smaller than the *_workspace query says            */
  ROAST_ERR_HIP = 5,         /* the HIP runtime refused a launch                                 */
  ROAST_ERR_UNSUPPORTED = 6  /* combination not implemented                                      */
} roast_status;

typedef enum { ROAST_F32 = 0, ROAST_BF16 = 1 } roast_dtype;

/* How colliding contributions to one slot of dM are summed.
 * ATOMIC: fp32 atomic adds, order varies from run to run.
 * DETERMINISTIC: per-block products go to the workspace and every slot is then summed in a fixed
 * order; the result is bit-identical from run to run. */
typedef enum { ROAST_REDUCE_ATOMIC = 0, ROAST_REDUCE_DETERMINISTIC = 1 } roast_reduce_mode;

/*
 * Hash parameters.  The paper asks only for universal hash functions h1 / h2 with range
 * {0, ..., |M| - block} and an independent sign hash g (Section 4.1); this library uses the
 * Carter-Wegman multiply-add family over a prime P on the 3-part key (k0, k1, k2):
 *
 *     u      = ((a0*(k0 mod P)) mod P + (a1*(k1 mod P)) mod P + (a2*(k2 mod P)) mod P + a3) mod P
 *     offset = align * (u mod (floor((|M| - block) / align) + 1))
 *     v      = the same form with s0..s3
 *     sign   = 1 - 2*(v & 1)
 *
 * use_sign = 0: no sign (+1 everywhere).  use_sign = 1: one sign per block (tile or chunk), v keyed
 * like the offset -- the reading this library takes as the default, and the one its fast kernels
 * implement.  use_sign = 2: one sign per element, v keyed by the element's own coordinates
 * ((layer_id, i, j) for W[i,j]; (table_id, row, d) for element d of a looked-up row), the form the
 * analysis of Section 5 uses; this variant runs on the generic kernels.  Other values:
 * ROAST_ERR_RANGE.
 *
 * ROAST-MM keys: (layer_id, x, y) with x the tile row (along H) and y the tile column (along O),
 * block = Z1*Z2.  Lookup keys: (table_id, row, chunk), block = Z.  Modules get independent hash
 * functions (Section 4.1 asks for that) by giving each module its own k0.
 * Requirements: 2 <= P < 2^32, every coefficient < P, align >= 1; otherwise ROAST_ERR_RANGE.
 */
typedef struct {
  uint64_t P;
  uint64_t a0, a1, a2, a3;
  uint64_t s0, s1, s2, s3;
  uint32_t use_sign;
  uint32_t align;
} roast_hash;

/* One ROAST-MM layer: virtual W is H x O (fan-in x fan-out) in Z1 x Z2 tiles; the tile grid is
 * ceil(H/Z1) x ceil(O/Z2); edge tiles keep the full Z2 row stride and the full offset range, their
 * elements outside H x O are never referenced.
 *   W[i, j] = lambda * sign(x, y) * M[offset(x, y) + Z2*(i mod Z1) + (j mod Z2)],  x = i/Z1, y = j/Z2
 * m_size is |M| in scalars. */
typedef struct {
  int64_t H, O;
  int32_t Z1, Z2;
  int64_t m_size;
  uint32_t layer_id;
  float lambda;
  roast_hash hash;
} roast_mm_desc;

/* One lookup module: rows of D scalars recovered in chunks of Z (the last chunk of a row is short
 * when Z does not divide D, but is still hashed into {0..|M|-Z}); chunks never straddle rows.
 *   out[n, i] = lambda * sign(t, r, c) * M[offset(t, r, c) + (i mod Z)],  c = i/Z, r = rows[n], t = table_ids[n] */
typedef struct {
  int64_t D;
  int32_t Z;
  int64_t m_size;
  float lambda;
  roast_hash hash;
} roast_embed_desc;

/* Human-readable name of a status code (static storage). */
const char* roast_status_string(roast_status s);

/*
 * Tile -> (offset, sign) map of one layer: the hash h2 and sign g of Section 4.1 evaluated on the
 * whole ceil(H/Z1) x ceil(O/Z2) grid, on the HOST with the same integer code the kernels use.
 * off_host / sgn_host: HOST arrays of ntx*nty entries, row-major in (x, y); either may be NULL.
 */
roast_status roast_tile_index(const roast_mm_desc* d, int64_t* off_host, int8_t* sgn_host);

/* The same map computed by the device code path, one thread per tile, into DEVICE arrays
 * (used to prove that host and device integer code agree bit for bit). */
roast_status roast_tile_index_device(const roast_mm_desc* d, int64_t* off_dev, int8_t* sgn_dev, void* stream);

/* Chunk -> (offset, sign) of N lookups on the device: off_dev / sgn_dev hold N*ceil(D/Z) entries,
 * entry n*ceil(D/Z) + c for chunk c of lookup n (the hash h1 of Section 4.1). */
roast_status roast_chunk_index_device(const roast_embed_desc* d, int64_t N, const int64_t* rows,
                                      const uint32_t* table_ids, int64_t* off_dev, int8_t* sgn_dev, void* stream);

/*
 * bf16 shadow of M (round to nearest even), about |M|-sized -- never |W|-sized.  Optional: the bf16
 * kernels stage the weight operand in bfloat16 anyway (see the conventions above), so reading it
 * from this copy gives bit-identical results with half the weight traffic.  Make it once per update
 * of M and pass it to as many roast_mm_fwd / roast_mm_bwd_dx calls as share that M.
 * The buffer holds two copies, the second shifted by one element, so that a tile at an odd offset
 * can be read with dword-aligned loads as well; its layout is private to the library.
 * shadow: DEVICE buffer of roast_m_shadow_bytes(m_size) bytes, 16-byte aligned, owned by the caller.
 */
size_t roast_m_shadow_bytes(int64_t m_size);
roast_status roast_m_shadow_bf16(const float* M, int64_t m_size, void* shadow, void* stream);

/*
 * ROAST-MM forward, Algorithm 1:  Y[I x O] = X[I x H] * W,  W recovered tile by tile from M.
 * X: I x H (ldx), Y: I x O (ldy), both of type `dt`; M: m_size fp32.  Y is overwritten.
 * M_bf16: NULL, or the shadow of this M made by roast_m_shadow_bf16 (used by the bf16 kernels only).
 */
roast_status roast_mm_fwd(const roast_mm_desc* d, roast_dtype dt, int64_t I, const void* X, int64_t ldx,
                          const float* M, const void* M_bf16, void* Y, int64_t ldy, void* stream);

/*
 * Gradient w.r.t. the input (Section 4.3):  dX[I x H] = dY[I x O] * W^T, W recovered from M.
 * dX is overwritten.  M_bf16 as for roast_mm_fwd.
 */
roast_status roast_mm_bwd_dx(const roast_mm_desc* d, roast_dtype dt, int64_t I, const void* dY, int64_t ldy,
                             const float* M, const void* M_bf16, void* dX, int64_t ldx, void* stream);

/*
 * Workspace variants of the two products above.  What the workspace buys depends on `dt`:
 *  - bf16, small batch (Algorithm 1's blocked product; the square-weight timings of Section 6 use batch
 *    512): with few rows the output has too few tiles to fill the chip, so the contraction axis is
 *    split over workgroups; each writes an fp32 partial output to the workspace and a second pass
 *    sums the parts in a fixed order and rounds once to bf16.
 *  - fp32: the product runs on the bf16 matrix cores.  X (or dY) and M are each held in the
 *    workspace as three bfloat16 planes with x = hi + mid + lo exactly, and the six plane products of
 *    weight >= 2^-16 are accumulated in fp32; the three dropped products -- (mid,lo), (lo,mid),
 *    (lo,lo) -- are bounded by 2^-21 |x||w| per term in the worst case (planes are truncated, so
 *    |mid| < 2^-7 |x| and |lo| < 2^-14 |x|) and are about 2^-24 |x||w| for typical mantissas: inside
 *    the fp32 bar of the conventions above.  Without a workspace fp32 runs on the vector ALUs.
 * The *_workspace queries return the bytes that help for these sizes (0: nothing to gain, or a
 * shape the matrix-core kernels do not cover; the plain call is used).
 * workspace: NULL (same as the plain call), or a DEVICE buffer, 16-byte aligned, of at least the
 * queried size (else ROAST_ERR_WORKSPACE); its contents are scratch, owned by the caller, and may be
 * reused by the next call on the same stream.  Results are deterministic for a fixed shape.
 */
/*
 * fp32 calls only: the three bfloat16 planes of M (each in the layout of the bf16 shadow), made once
 * per update of M and passed as `M_bf16` to fp32 roast_mm_fwd_ws / roast_mm_bwd_dx_ws calls, which
 * otherwise rebuild them in their workspace on every call (a pass over |M|).
 * NOTE: the `M_bf16` argument therefore names a different buffer per dtype -- ROAST_BF16 calls take
 * the shadow (roast_m_shadow_bytes), ROAST_F32 calls with a workspace take the planes
 * (roast_m_planes_bytes, three times as large).  The C-ABI carries no size for it and cannot tell
 * them apart: passing a shadow to an fp32 call makes the kernels read past its end.  NULL is always
 * safe.
 * planes: DEVICE buffer of roast_m_planes_bytes(m_size) bytes, 16-byte aligned, owned by the caller.
 */
size_t roast_m_planes_bytes(int64_t m_size);
roast_status roast_m_planes_bf16(const float* M, int64_t m_size, void* planes, void* stream);

size_t roast_mm_fwd_workspace(const roast_mm_desc* d, roast_dtype dt, int64_t I);
size_t roast_mm_bwd_dx_workspace(const roast_mm_desc* d, roast_dtype dt, int64_t I);
roast_status roast_mm_fwd_ws(const roast_mm_desc* d, roast_dtype dt, int64_t I, const void* X, int64_t ldx,
                             const float* M, const void* M_bf16, void* Y, int64_t ldy, void* workspace,
                             size_t workspace_bytes, void* stream);
roast_status roast_mm_bwd_dx_ws(const roast_mm_desc* d, roast_dtype dt, int64_t I, const void* dY, int64_t ldy,
                                const float* M, const void* M_bf16, void* dX, int64_t ldx, void* workspace,
                                size_t workspace_bytes, void* stream);

/*
 * Diagnostic, host only, launches nothing: how many consecutive 128-column output blocks one
 * workgroup of the bf16 matrix-core kernels computes, one after the other as a single run of
 * contraction steps, in roast_mm_fwd (which = 0) or roast_mm_bwd_dx (which = 1) on I rows with a
 * bf16 shadow and no workspace.  This is Algorithm 1's loop order seen from one workgroup: a fixed
 * row block i, the column blocks j of its strip in turn, the contraction k innermost.  1 = one block
 * per workgroup (also for shapes that take other kernels); 0 = invalid descriptor, I or `which`.
 * For tests (which must know that a shape exercises the strip path) and for tuning.
 */
int roast_mm_strip_blocks(const roast_mm_desc* d, int64_t I, int which);

/* Bytes of workspace roast_mm_bwd_dM can use for these sizes and mode (0 = none).
 * DETERMINISTIC: required.  ATOMIC: optional -- with it (bf16 path, contraction split over several
 * workgroups) the per-split products are summed in the workspace and scattered with one atomic per
 * virtual weight; without it every split adds straight into dM. */
size_t roast_mm_bwd_dM_workspace(const roast_mm_desc* d, int64_t I, roast_reduce_mode mode);
/* fp32, ATOMIC mode only: bytes of the optional workspace with which roast_mm_bwd_dM runs the product
 * on the matrix cores from bfloat16 planes of X and dY (see roast_mm_fwd_ws); 0 = shape not covered. */
size_t roast_mm_bwd_dM_workspace_f32(const roast_mm_desc* d, int64_t I);

/*
 * Gradient w.r.t. the shared array (Section 4.3 gradient equation, Appendix A.1):
 *   dM[offset(x,y) + Z2*o1 + o2] += lambda * sign(x,y) * sum_i X[i, x*Z1+o1] * dY[i, y*Z2+o2]
 * for every element of every tile; colliding tiles add up.  dM: m_size fp32, accumulated into.
 * ws / ws_bytes: device scratch of at least roast_mm_bwd_dM_workspace() bytes (may be NULL / 0
 * when that is 0 or, in ATOMIC mode, always); its contents on return are unspecified.
 */
roast_status roast_mm_bwd_dM(const roast_mm_desc* d, roast_dtype dt, int64_t I,
                             const void* X, int64_t ldx, const void* dY, int64_t ldy,
                             float* dM, roast_reduce_mode mode, void* ws, size_t ws_bytes, void* stream);

/*
 * Lookup L(l, W) of Section 4.1 for N ids at once: out[N x D] fp32 (dense, row stride D),
 * rows: N int64 row ids (>= 0), table_ids: N uint32 (first hash key of each lookup).
 */
roast_status roast_embed_fwd(const roast_embed_desc* d, int64_t N, const int64_t* rows,
                             const uint32_t* table_ids, const float* M, float* out, void* stream);

/* Bytes of workspace roast_embed_bwd can use for these sizes and mode (0 = none).
 * ATOMIC: optional -- with it, large batches are first routed by destination (per-bucket lists in
 * the workspace) and summed in on-chip memory before they touch dM; without it every element is an
 * fp32 atomic add into dM.  DETERMINISTIC: required. */
size_t roast_embed_bwd_workspace(const roast_embed_desc* d, int64_t N, roast_reduce_mode mode);

/*
 * Gradient of the lookup (Section 4.3):  dM[offset(t,r,c) + o] += lambda * sign * dOut[n, c*Z + o].
 * dOut: N x D fp32 (row stride D); dM: m_size fp32, accumulated into.
 * DETERMINISTIC: every product fl(lambda * sign * dOut[..]) is converted to 64-bit fixed point with a
 * quantum derived from the largest |dOut| of the call (at least 31 bits below it), summed with
 * integer atomics -- exact, hence independent of the order -- and added to dM with one rounding per
 * slot; bit-identical from run to run.  dOut must be finite (an Inf or NaN turns all of dM into NaN).
 * ws / ws_bytes: device scratch of at least roast_embed_bwd_workspace() bytes (may be NULL / 0 in
 * ATOMIC mode); its contents on return are unspecified.
 */
roast_status roast_embed_bwd(const roast_embed_desc* d, int64_t N, const int64_t* rows,
                             const uint32_t* table_ids, const float* dOut, float* dM,
                             roast_reduce_mode mode, void* ws, size_t ws_bytes, void* stream);

/*
 * roast_embed_bwd for callers that cannot allocate device memory and have no buffer to lend: code
 * under HIP graph capture, tight serving / training loops with a fixed memory plan, harnesses that
 * forbid hipMalloc.  Same arguments and results as roast_embed_bwd (both modes, same kernels), but
 * the workspace is a 64 MiB array inside the library's code object instead of `ws`: the call neither
 * allocates nor frees (no hipMalloc / hipFree, no allocating library routine) and takes no scratch.
 *   - Limit: the bytes roast_embed_bwd_workspace(d, N, mode) reports must not exceed 64 MiB
 *     (67 108 864); beyond that the call returns ROAST_ERR_WORKSPACE and launches nothing.  (ATOMIC:
 *     about 16 bytes per chunk of the batch + 64 KiB per 4096 slots of M; DETERMINISTIC adds 8 bytes
 *     per slot of M.  Config-4-sized M: up to ~690 000 lookups of 4 chunks per call.)
 *   - Each GPU holds its own copy of the array from the moment the library's code is loaded on it
 *     until the process ends.  The first call on a device looks its address up (once per device; do
 *     that first call outside a graph capture, like every kernel's first launch).
 *   - All calls on one GPU share that GPU's array, and it keeps the previous call's contents: the
 *     call clears what must start at zero with fill kernels on `stream`.  Two such calls that overlap
 *     in time on one GPU (different streams, or different host threads without ordering) race on the
 *     array and give wrong gradients; calls ordered on one stream are safe.
 */
roast_status roast_embed_bwd_noalloc(const roast_embed_desc* d, int64_t N, const int64_t* rows,
                                     const uint32_t* table_ids, const float* dOut, float* dM,
                                     roast_reduce_mode mode, void* stream);

/*
 * Pooled (bag-sum) lookup: the lookup L of Section 4.1 applied to every id of a bag, summed per bag
 * (the multi-hot use of an embedding table):
 *   out[b, :] = sum over n in [bag_offsets[b], bag_offsets[b+1]) of the row roast_embed_fwd returns
 *               for (rows[n], table_ids[n]);   out: B x D fp32 (row stride D), overwritten.
 * bag_offsets: DEVICE array of B + 1 int64: bag_offsets[0] = 0, non-decreasing, bag_offsets[B] = N;
 * an empty bag gives a zero row.  The library cannot check device data: offsets that break the
 * contract give unspecified values in `out` / `dM`, but every access stays inside the arrays.
 * Sums run in lookup order: results are bit-reproducible.
 */
roast_status roast_embed_bag_fwd(const roast_embed_desc* d, int64_t N, int64_t B, const int64_t* rows,
                                 const uint32_t* table_ids, const int64_t* bag_offsets, const float* M,
                                 float* out, void* stream);

/* Workspace of roast_embed_bag_bwd; same meaning as roast_embed_bwd_workspace. */
size_t roast_embed_bag_bwd_workspace(const roast_embed_desc* d, int64_t N, int64_t B, roast_reduce_mode mode);

/*
 * Gradient of the pooled lookup (Section 4.3 applied to a sum: every lookup of bag b receives
 * dOut[b, :]):  dM[offset(t,r,c) + o] += lambda * sign * dOut[bag(n), c*Z + o]  for all n.
 * dOut: B x D fp32 (row stride D); dM, mode, ws / ws_bytes as for roast_embed_bwd.
 */
roast_status roast_embed_bag_bwd(const roast_embed_desc* d, int64_t N, int64_t B, const int64_t* rows,
                                 const uint32_t* table_ids, const int64_t* bag_offsets, const float* dOut,
                                 float* dM, roast_reduce_mode mode, void* ws, size_t ws_bytes, void* stream);

/*
 * Optimizer step on the shared array: the "update weights" leg of the paper's training workload
 * (training-time tables of the appendix: SGD, Adagrad, Adam on the |M|-sized parameter).  The paper
 * defines no update rule of its own; these are the textbook rules in the form of the stock optimizers:
 *   g = dM + weight_decay * M
 *   SGD     : M -= lr * g
 *   ADAGRAD : state1 += g*g ;  M -= lr * g / (sqrt(state1) + eps)
 *   ADAM    : state1 = beta1*state1 + (1-beta1)*g ;  state2 = beta2*state2 + (1-beta2)*g*g ;
 *             M -= lr * (state1 / (1 - beta1^step)) / (sqrt(state2 / (1 - beta2^step)) + eps)
 * `step` is the 1-based count of this update (Adam only).  zero_grad != 0 clears dM in the same pass.
 */
typedef enum { ROAST_OPT_SGD = 0, ROAST_OPT_ADAGRAD = 1, ROAST_OPT_ADAM = 2 } roast_optimizer;

typedef struct {
  roast_optimizer kind;
  float lr, weight_decay;
  float beta1, beta2, eps;
  int64_t step;
  uint32_t zero_grad;
} roast_optim_desc;

/*
 * One pass over m_size parameters.  M, dM: m_size fp32, both updated in place (dM only when
 * zero_grad).  state1: m_size fp32 for ADAGRAD and ADAM, state2: m_size fp32 for ADAM (the caller
 * zeroes them before the first step); ignored (may be NULL) otherwise.  M_bf16: NULL, or a shadow
 * buffer as for roast_m_shadow_bf16, refreshed from the new M in the same pass.
 * All pointers are DEVICE pointers, 16-byte aligned.  ROAST_ERR_ARG: null M / dM / needed state,
 * misaligned pointer, bad kind, step < 1 for ADAM, beta outside [0, 1).
 */
roast_status roast_optim_step(const roast_optim_desc* d, int64_t m_size, float* M, float* dM, float* state1,
                              float* state2, void* M_bf16, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* ROAST_H */
