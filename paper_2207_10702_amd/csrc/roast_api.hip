// C-ABI entry points: argument validation on the host, then dispatch to the kernels.
// Nothing here allocates device memory or synchronises.
#include "roast.h"
#include "roast_internal.hpp"

using namespace roast;

namespace {

roast_status check_hash(const roast_hash& h) {
  if (h.P < 2 || h.P >= (1ull << 32) || h.align < 1 || h.use_sign > 2) return ROAST_ERR_RANGE;
  const uint64_t c[8] = {h.a0, h.a1, h.a2, h.a3, h.s0, h.s1, h.s2, h.s3};
  for (uint64_t v : c)
    if (v >= h.P) return ROAST_ERR_RANGE;
  return ROAST_OK;
}

roast_status make_mm_args(const roast_mm_desc* d, int64_t I, MMArgs* a) {
  if (!d || I < 0) return ROAST_ERR_ARG;
  if (d->H <= 0 || d->O <= 0 || d->Z1 <= 0 || d->Z2 <= 0) return ROAST_ERR_SHAPE;
  if (d->H >= (1ll << 31) || d->O >= (1ll << 31) || I >= (1ll << 31)) return ROAST_ERR_UNSUPPORTED;
  const int64_t L = (int64_t)d->Z1 * d->Z2;
  if (d->m_size < L) return ROAST_ERR_RANGE;
  roast_status st = check_hash(d->hash);
  if (st != ROAST_OK) return st;
  a->I = I; a->H = d->H; a->O = d->O; a->Z1 = d->Z1; a->Z2 = d->Z2;
  a->nTx = (d->H + d->Z1 - 1) / d->Z1;
  a->nTy = (d->O + d->Z2 - 1) / d->Z2;
  a->m_size = d->m_size;
  a->layer = d->layer_id;
  a->lambda = d->lambda;
  a->hash = make_hash_dev(d->hash, d->m_size, L);
  return ROAST_OK;
}

roast_status make_embed_args(const roast_embed_desc* d, int64_t N, EmbedArgs* a) {
  if (!d || N < 0) return ROAST_ERR_ARG;
  if (d->D <= 0 || d->Z <= 0) return ROAST_ERR_SHAPE;
  if (d->D >= (1ll << 31)) return ROAST_ERR_UNSUPPORTED;
  if (d->m_size < d->Z) return ROAST_ERR_RANGE;
  roast_status st = check_hash(d->hash);
  if (st != ROAST_OK) return st;
  a->N = N; a->D = d->D; a->Z = d->Z;
  a->C = (d->D + d->Z - 1) / d->Z;
  a->m_size = d->m_size;
  a->lambda = d->lambda;
  a->hash = make_hash_dev(d->hash, d->m_size, d->Z);
  a->bag_off = nullptr;
  a->B = 0;
  return ROAST_OK;
}

bool dtype_ok(roast_dtype dt) { return dt == ROAST_F32 || dt == ROAST_BF16; }
bool mode_ok(roast_reduce_mode m) { return m == ROAST_REDUCE_ATOMIC || m == ROAST_REDUCE_DETERMINISTIC; }

}  // namespace

// The runtime keeps the last error of ANY earlier HIP call of the process (the caller's own, or a
// framework's probe that is expected to fail) until somebody reads it; an entry point that launches
// kernels drops it first, so that the status it returns is about its own launches.
static inline void drop_stale_error() { (void)hipGetLastError(); }

extern "C" {

const char* roast_status_string(roast_status s) {
  switch (s) {
    case ROAST_OK: return "ok";
    case ROAST_ERR_ARG: return "bad argument (null pointer, negative size, leading dimension too small or bad enum)";
    case ROAST_ERR_SHAPE: return "bad shape (H, O, Z1, Z2, D and Z must be positive)";
    case ROAST_ERR_RANGE: return "block does not fit in M or hash parameters out of range";
    case ROAST_ERR_WORKSPACE: return "workspace missing or too small";
    case ROAST_ERR_HIP: return "HIP runtime error";
    case ROAST_ERR_UNSUPPORTED: return "unsupported combination";
  }
  return "unknown status";
}

roast_status roast_tile_index(const roast_mm_desc* d, int64_t* off_host, int8_t* sgn_host) {
  MMArgs a;
  roast_status st = make_mm_args(d, 0, &a);
  if (st != ROAST_OK) return st;
  for (int64_t x = 0; x < a.nTx; ++x)
    for (int64_t y = 0; y < a.nTy; ++y) {
      if (off_host) off_host[x * a.nTy + y] = block_offset(a.hash, a.layer, (uint64_t)x, (uint64_t)y);
      if (sgn_host) sgn_host[x * a.nTy + y] = (int8_t)block_sign(a.hash, a.layer, (uint64_t)x, (uint64_t)y);
    }
  return ROAST_OK;
}

roast_status roast_tile_index_device(const roast_mm_desc* d, int64_t* off_dev, int8_t* sgn_dev, void* stream) {
  drop_stale_error();
  MMArgs a;
  roast_status st = make_mm_args(d, 0, &a);
  if (st != ROAST_OK) return st;
  if (!off_dev || !sgn_dev) return ROAST_ERR_ARG;
  return tile_index_launch(a, off_dev, sgn_dev, (hipStream_t)stream);
}

roast_status roast_chunk_index_device(const roast_embed_desc* d, int64_t N, const int64_t* rows,
                                      const uint32_t* table_ids, int64_t* off_dev, int8_t* sgn_dev, void* stream) {
  drop_stale_error();
  EmbedArgs a;
  roast_status st = make_embed_args(d, N, &a);
  if (st != ROAST_OK) return st;
  if (N == 0) return ROAST_OK;
  if (!rows || !table_ids || !off_dev || !sgn_dev) return ROAST_ERR_ARG;
  return chunk_index_launch(a, rows, table_ids, off_dev, sgn_dev, (hipStream_t)stream);
}

size_t roast_m_shadow_bytes(int64_t m_size) {
  return m_size > 0 ? (size_t)(2 * shadow_stride(m_size)) * 2 : 0;
}

size_t roast_m_planes_bytes(int64_t m_size) { return m_size > 0 ? m_planes_bytes(m_size) : 0; }

roast_status roast_m_planes_bf16(const float* M, int64_t m_size, void* planes, void* stream) {
  drop_stale_error();
  if (m_size < 0) return ROAST_ERR_ARG;
  if (m_size == 0) return ROAST_OK;
  if (!M || !planes || ((uintptr_t)planes & 15) != 0) return ROAST_ERR_ARG;
  return m_planes_launch(M, m_size, planes, (hipStream_t)stream);
}

roast_status roast_m_shadow_bf16(const float* M, int64_t m_size, void* shadow, void* stream) {
  drop_stale_error();
  if (m_size < 0) return ROAST_ERR_ARG;
  if (m_size == 0) return ROAST_OK;
  if (!M || !shadow || ((uintptr_t)shadow & 15) != 0) return ROAST_ERR_ARG;
  return shadow_bf16_launch(M, m_size, shadow, (hipStream_t)stream);
}

size_t roast_mm_fwd_workspace(const roast_mm_desc* d, roast_dtype dt, int64_t I) {
  MMArgs a;
  if (make_mm_args(d, I, &a) != ROAST_OK || !dtype_ok(dt) || I == 0) return 0;
  if (dt == ROAST_F32) return x3_fwd_workspace(a);
  const int s = mfma_fwd_splits(a);
  return s > 1 ? (size_t)s * (size_t)I * (size_t)a.O * sizeof(float) : 0;
}

size_t roast_mm_bwd_dx_workspace(const roast_mm_desc* d, roast_dtype dt, int64_t I) {
  MMArgs a;
  if (make_mm_args(d, I, &a) != ROAST_OK || !dtype_ok(dt) || I == 0) return 0;
  if (dt == ROAST_F32) return x3_dx_workspace(a);
  const int s = mfma_dx_splits(a);
  return s > 1 ? (size_t)s * (size_t)I * (size_t)a.H * sizeof(float) : 0;
}

int roast_mm_strip_blocks(const roast_mm_desc* d, int64_t I, int which) {
  MMArgs a;
  if (make_mm_args(d, I, &a) != ROAST_OK || I <= 0 || (which != 0 && which != 1)) return 0;
  return which == 0 ? mfma_fwd_strip(a, true) : mfma_dx_strip(a, true);
}

roast_status roast_mm_fwd_ws(const roast_mm_desc* d, roast_dtype dt, int64_t I, const void* X, int64_t ldx,
                             const float* M, const void* M_bf16, void* Y, int64_t ldy, void* workspace,
                             size_t workspace_bytes, void* stream) {
  drop_stale_error();
  MMArgs a;
  roast_status st = make_mm_args(d, I, &a);
  if (st != ROAST_OK) return st;
  if (!dtype_ok(dt)) return ROAST_ERR_ARG;
  if (I == 0) return ROAST_OK;
  if (!X || !M || !Y || ldx < a.H || ldy < a.O) return ROAST_ERR_ARG;
  if (dt == ROAST_BF16) {
    const size_t need = roast_mm_fwd_workspace(d, dt, I);
    if (workspace && (workspace_bytes < need || ((uintptr_t)workspace & 15) != 0)) return ROAST_ERR_WORKSPACE;
    st = mfma_mm_fwd(a, X, ldx, M, M_bf16, Y, ldy, need ? (float*)workspace : nullptr, (hipStream_t)stream);
    if (st != ROAST_ERR_UNSUPPORTED) return st;
  } else if (workspace) {
    const size_t need = roast_mm_fwd_workspace(d, dt, I);
    if (workspace_bytes < need || ((uintptr_t)workspace & 15) != 0) return ROAST_ERR_WORKSPACE;
    if (need) {
      st = x3_mm_fwd(a, (const float*)X, ldx, M, M_bf16, (float*)Y, ldy, workspace, (hipStream_t)stream);
      if (st != ROAST_ERR_UNSUPPORTED) return st;
    }
  }
  return generic_mm_fwd(a, dt, X, ldx, M, Y, ldy, (hipStream_t)stream);
}

roast_status roast_mm_fwd(const roast_mm_desc* d, roast_dtype dt, int64_t I, const void* X, int64_t ldx,
                          const float* M, const void* M_bf16, void* Y, int64_t ldy, void* stream) {
  return roast_mm_fwd_ws(d, dt, I, X, ldx, M, M_bf16, Y, ldy, nullptr, 0, stream);
}

roast_status roast_mm_bwd_dx_ws(const roast_mm_desc* d, roast_dtype dt, int64_t I, const void* dY, int64_t ldy,
                                const float* M, const void* M_bf16, void* dX, int64_t ldx, void* workspace,
                                size_t workspace_bytes, void* stream) {
  drop_stale_error();
  MMArgs a;
  roast_status st = make_mm_args(d, I, &a);
  if (st != ROAST_OK) return st;
  if (!dtype_ok(dt)) return ROAST_ERR_ARG;
  if (I == 0) return ROAST_OK;
  if (!dY || !M || !dX || ldx < a.H || ldy < a.O) return ROAST_ERR_ARG;
  if (dt == ROAST_BF16) {
    const size_t need = roast_mm_bwd_dx_workspace(d, dt, I);
    if (workspace && (workspace_bytes < need || ((uintptr_t)workspace & 15) != 0)) return ROAST_ERR_WORKSPACE;
    st = mfma_mm_bwd_dx(a, dY, ldy, M, M_bf16, dX, ldx, need ? (float*)workspace : nullptr, (hipStream_t)stream);
    if (st != ROAST_ERR_UNSUPPORTED) return st;
  } else if (workspace) {
    const size_t need = roast_mm_bwd_dx_workspace(d, dt, I);
    if (workspace_bytes < need || ((uintptr_t)workspace & 15) != 0) return ROAST_ERR_WORKSPACE;
    if (need) {
      st = x3_mm_bwd_dx(a, (const float*)dY, ldy, M, M_bf16, (float*)dX, ldx, workspace, (hipStream_t)stream);
      if (st != ROAST_ERR_UNSUPPORTED) return st;
    }
  }
  return generic_mm_bwd_dx(a, dt, dY, ldy, M, dX, ldx, (hipStream_t)stream);
}

roast_status roast_mm_bwd_dx(const roast_mm_desc* d, roast_dtype dt, int64_t I, const void* dY, int64_t ldy,
                             const float* M, const void* M_bf16, void* dX, int64_t ldx, void* stream) {
  return roast_mm_bwd_dx_ws(d, dt, I, dY, ldy, M, M_bf16, dX, ldx, nullptr, 0, stream);
}

size_t roast_mm_bwd_dM_workspace_f32(const roast_mm_desc* d, int64_t I) {
  MMArgs a;
  if (make_mm_args(d, I, &a) != ROAST_OK || I == 0) return 0;
  return x3_dm_workspace(a);
}

size_t roast_mm_bwd_dM_workspace(const roast_mm_desc* d, int64_t I, roast_reduce_mode mode) {
  MMArgs a;
  if (make_mm_args(d, I, &a) != ROAST_OK) return 0;
  if (I == 0) return 0;
  return mode == ROAST_REDUCE_DETERMINISTIC ? dm_det_workspace_bytes(a) : dm_ws_workspace_bytes(a);
}

roast_status roast_mm_bwd_dM(const roast_mm_desc* d, roast_dtype dt, int64_t I, const void* X, int64_t ldx,
                             const void* dY, int64_t ldy, float* dM, roast_reduce_mode mode, void* ws,
                             size_t ws_bytes, void* stream) {
  drop_stale_error();
  MMArgs a;
  roast_status st = make_mm_args(d, I, &a);
  if (st != ROAST_OK) return st;
  if (!dtype_ok(dt) || !mode_ok(mode)) return ROAST_ERR_ARG;
  if (I == 0) return ROAST_OK;
  if (!X || !dY || !dM || ldx < a.H || ldy < a.O) return ROAST_ERR_ARG;
  if (mode == ROAST_REDUCE_DETERMINISTIC) {
    const size_t need = dm_det_workspace_bytes(a);
    if (need == 0) return ROAST_ERR_UNSUPPORTED;
    if (!ws || ws_bytes < need) return ROAST_ERR_WORKSPACE;
    return dm_det_run(a, dt, X, ldx, dY, ldy, dM, ws, (hipStream_t)stream);
  }
  if (dt == ROAST_BF16) {
    // optional workspace: per-split products are summed before they are scattered (fewer atomics)
    const size_t want = dm_ws_workspace_bytes(a);
    if (want && ws && ws_bytes >= want) {
      st = dm_ws_run(a, X, ldx, dY, ldy, dM, ws, (hipStream_t)stream);
      if (st != ROAST_ERR_UNSUPPORTED) return st;
    }
    st = mfma_mm_bwd_dM(a, X, ldx, dY, ldy, dM, nullptr, 0, (hipStream_t)stream);
    if (st != ROAST_ERR_UNSUPPORTED) return st;
  } else {
    // optional workspace: the product runs on the matrix cores from bfloat16 planes of X and dY
    const size_t want = x3_dm_workspace(a);
    if (want && ws && ws_bytes >= want && ((uintptr_t)ws & 15) == 0) {
      st = x3_mm_bwd_dM(a, (const float*)X, ldx, (const float*)dY, ldy, dM, ws, (hipStream_t)stream);
      if (st != ROAST_ERR_UNSUPPORTED) return st;
    }
  }
  return generic_mm_bwd_dM_atomic(a, dt, X, ldx, dY, ldy, dM, (hipStream_t)stream);
}

roast_status roast_embed_fwd(const roast_embed_desc* d, int64_t N, const int64_t* rows, const uint32_t* table_ids,
                             const float* M, float* out, void* stream) {
  drop_stale_error();
  EmbedArgs a;
  roast_status st = make_embed_args(d, N, &a);
  if (st != ROAST_OK) return st;
  if (N == 0) return ROAST_OK;
  if (!rows || !table_ids || !M || !out) return ROAST_ERR_ARG;
  return embed_fwd_launch(a, rows, table_ids, M, out, (hipStream_t)stream);
}

size_t roast_embed_bwd_workspace(const roast_embed_desc* d, int64_t N, roast_reduce_mode mode) {
  EmbedArgs a;
  if (make_embed_args(d, N, &a) != ROAST_OK) return 0;
  if (N == 0) return 0;
  return mode == ROAST_REDUCE_DETERMINISTIC ? embed_det_workspace_bytes(a) : embed_bucket_workspace_bytes(a);
}

roast_status roast_embed_bwd(const roast_embed_desc* d, int64_t N, const int64_t* rows, const uint32_t* table_ids,
                             const float* dOut, float* dM, roast_reduce_mode mode, void* ws, size_t ws_bytes,
                             void* stream) {
  drop_stale_error();
  EmbedArgs a;
  roast_status st = make_embed_args(d, N, &a);
  if (st != ROAST_OK) return st;
  if (!mode_ok(mode)) return ROAST_ERR_ARG;
  if (N == 0) return ROAST_OK;
  if (!rows || !table_ids || !dOut || !dM) return ROAST_ERR_ARG;
  if (mode == ROAST_REDUCE_DETERMINISTIC) {
    const size_t need = embed_det_workspace_bytes(a);
    if (need == 0) return ROAST_ERR_UNSUPPORTED;
    if (!ws || ws_bytes < need) return ROAST_ERR_WORKSPACE;
    return embed_bwd_det_run(a, rows, table_ids, dOut, dM, ws, (hipStream_t)stream);
  }
  return embed_bwd_atomic_launch(a, rows, table_ids, dOut, dM, ws, ws_bytes, (hipStream_t)stream);
}

roast_status roast_embed_bwd_noalloc(const roast_embed_desc* d, int64_t N, const int64_t* rows,
                                     const uint32_t* table_ids, const float* dOut, float* dM,
                                     roast_reduce_mode mode, void* stream) {
  drop_stale_error();
  EmbedArgs a;
  roast_status st = make_embed_args(d, N, &a);
  if (st != ROAST_OK) return st;
  if (!mode_ok(mode)) return ROAST_ERR_ARG;
  if (N == 0) return ROAST_OK;
  if (!rows || !table_ids || !dOut || !dM) return ROAST_ERR_ARG;
  return embed_bwd_static_run(a, rows, table_ids, dOut, dM, mode == ROAST_REDUCE_DETERMINISTIC, (hipStream_t)stream);
}

roast_status roast_embed_bag_fwd(const roast_embed_desc* d, int64_t N, int64_t B, const int64_t* rows,
                                 const uint32_t* table_ids, const int64_t* bag_offsets, const float* M, float* out,
                                 void* stream) {
  drop_stale_error();
  EmbedArgs a;
  roast_status st = make_embed_args(d, N, &a);
  if (st != ROAST_OK) return st;
  if (B < 0) return ROAST_ERR_ARG;
  if (B == 0) return ROAST_OK;
  if (!bag_offsets || !M || !out || (N > 0 && (!rows || !table_ids))) return ROAST_ERR_ARG;
  a.bag_off = bag_offsets;
  a.B = B;
  return embed_bag_fwd_launch(a, rows, table_ids, M, out, (hipStream_t)stream);
}

size_t roast_embed_bag_bwd_workspace(const roast_embed_desc* d, int64_t N, int64_t B, roast_reduce_mode mode) {
  EmbedArgs a;
  if (make_embed_args(d, N, &a) != ROAST_OK || B <= 0 || N == 0) return 0;
  a.B = B;
  return mode == ROAST_REDUCE_DETERMINISTIC ? embed_det_workspace_bytes(a) : embed_bucket_workspace_bytes(a);
}

roast_status roast_embed_bag_bwd(const roast_embed_desc* d, int64_t N, int64_t B, const int64_t* rows,
                                 const uint32_t* table_ids, const int64_t* bag_offsets, const float* dOut, float* dM,
                                 roast_reduce_mode mode, void* ws, size_t ws_bytes, void* stream) {
  drop_stale_error();
  EmbedArgs a;
  roast_status st = make_embed_args(d, N, &a);
  if (st != ROAST_OK) return st;
  if (!mode_ok(mode) || B < 0) return ROAST_ERR_ARG;
  if (N == 0 || B == 0) return ROAST_OK;
  if (!rows || !table_ids || !bag_offsets || !dOut || !dM) return ROAST_ERR_ARG;
  a.bag_off = bag_offsets;
  a.B = B;
  if (mode == ROAST_REDUCE_DETERMINISTIC) {
    const size_t need = embed_det_workspace_bytes(a);
    if (need == 0) return ROAST_ERR_UNSUPPORTED;
    if (!ws || ws_bytes < need) return ROAST_ERR_WORKSPACE;
    return embed_bwd_det_run(a, rows, table_ids, dOut, dM, ws, (hipStream_t)stream);
  }
  return embed_bwd_atomic_launch(a, rows, table_ids, dOut, dM, ws, ws_bytes, (hipStream_t)stream);
}

roast_status roast_optim_step(const roast_optim_desc* d, int64_t m_size, float* M, float* dM, float* state1,
                              float* state2, void* M_bf16, void* stream) {
  drop_stale_error();
  if (!d || m_size < 0) return ROAST_ERR_ARG;
  if (d->kind != ROAST_OPT_SGD && d->kind != ROAST_OPT_ADAGRAD && d->kind != ROAST_OPT_ADAM) return ROAST_ERR_ARG;
  if (d->kind == ROAST_OPT_ADAM &&
      (d->step < 1 || !(d->beta1 >= 0.f && d->beta1 < 1.f) || !(d->beta2 >= 0.f && d->beta2 < 1.f)))
    return ROAST_ERR_ARG;
  if (m_size == 0) return ROAST_OK;
  auto bad = [](const void* p) { return p == nullptr || ((uintptr_t)p & 15) != 0; };
  if (bad(M) || bad(dM)) return ROAST_ERR_ARG;
  if (d->kind != ROAST_OPT_SGD && bad(state1)) return ROAST_ERR_ARG;
  if (d->kind == ROAST_OPT_ADAM && bad(state2)) return ROAST_ERR_ARG;
  if (M_bf16 && ((uintptr_t)M_bf16 & 15) != 0) return ROAST_ERR_ARG;
  return optim_launch(*d, m_size, M, dM, state1, state2, M_bf16, (hipStream_t)stream);
}

}  // extern "C"
