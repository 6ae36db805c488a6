// The C ABI: argument validation (everything checkable on the host is rejected before any
// launch), workspace sizing, and dispatch to the four stages.  No device memory is allocated,
// freed or retained here, and no call synchronises.
#include <math.h>
#include <string.h>

#include "gvote_internal.hpp"

using namespace gvote;

namespace {

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

gvote_status check_shape(const gvote_shape *sh) {
  if (!sh) return GVOTE_ERR_INVALID_ARG;
  if (sh->dtype != GVOTE_F32 && sh->dtype != GVOTE_BF16) return GVOTE_ERR_UNSUPPORTED;
  if (sh->d_model < 8 || sh->n_q_heads < 1 || sh->n_kv_heads < 1 || sh->head_dim < 8) return GVOTE_ERR_SHAPE;
  if (sh->d_model % 8 || sh->head_dim % 8 || sh->n_q_heads % sh->n_kv_heads) return GVOTE_ERR_SHAPE;
  if (sh->head_dim > 256) return GVOTE_ERR_UNSUPPORTED;
  if (!(sh->rope_theta > 1.0f) || !isfinite(sh->rope_theta)) return GVOTE_ERR_INVALID_ARG;
  return GVOTE_OK;
}

enum Need { NEED_HIDDEN = 1, NEED_WQ = 2, NEED_K = 4, NEED_V = 8 };

gvote_status check_items(const gvote_shape *sh, const gvote_item *items, int32_t n_items, int need) {
  if (!items || n_items < 1) return GVOTE_ERR_INVALID_ARG;
  for (int i = 0; i < n_items; ++i) {
    const gvote_item &g = items[i];
    if (g.L < 2 || g.n_skip < 0 || g.n_skip > g.L - 2) return GVOTE_ERR_INVALID_ARG;
    if (g.n_future < 1 || g.n_future > 4096 || g.pos0 < 0) return GVOTE_ERR_INVALID_ARG;
    if (need & NEED_HIDDEN) {
      if (!g.hidden) return GVOTE_ERR_INVALID_ARG;
      if (!aligned16(g.hidden) || g.hidden_row_stride < sh->d_model || g.hidden_row_stride % 8) return GVOTE_ERR_SHAPE;
    }
    if (need & NEED_WQ) {
      if (!g.w_q) return GVOTE_ERR_INVALID_ARG;
      if (!aligned16(g.w_q) || (g.b_q && !aligned16(g.b_q))) return GVOTE_ERR_SHAPE;
    }
    if (need & (NEED_K | NEED_V)) {
      if (!g.k || ((need & NEED_V) && !g.v)) return GVOTE_ERR_INVALID_ARG;
      if (!aligned16(g.k) || ((need & NEED_V) && !aligned16(g.v))) return GVOTE_ERR_SHAPE;
      if (g.kv_head_stride < sh->head_dim || g.kv_head_stride % 8 || g.kv_tok_stride % 8) return GVOTE_ERR_SHAPE;
      if (g.kv_tok_stride < sh->head_dim) return GVOTE_ERR_SHAPE;
    }
  }
  return GVOTE_OK;
}

size_t max_sz(size_t a, size_t b) { return a > b ? a : b; }

size_t workspace_bytes_unchecked(const gvote_shape *sh, const gvote_item *items, int32_t n_items, int32_t S) {
  size_t w = plan_fit(sh, items, n_items).ws_bytes;
  w = max_sz(w, plan_sample(sh, n_items, S).ws_bytes);
  w = max_sz(w, plan_score(sh, items, n_items, S).ws_bytes);
  w = max_sz(w, plan_union(sh, items, n_items).ws_bytes);
  w = max_sz(w, overlap_ws_bytes(sh, items, n_items));
  w = max_sz(w, decode_ws_bytes(sh, n_items));
  return align_up(w, 256) + 256;
}

}  // namespace

extern "C" {

const char *gvote_status_string(gvote_status st) {
  switch (st) {
    case GVOTE_OK: return "ok";
    case GVOTE_ERR_INVALID_ARG: return "invalid argument";
    case GVOTE_ERR_SHAPE: return "inconsistent or misaligned shape, stride or pointer";
    case GVOTE_ERR_UNSUPPORTED: return "unsupported configuration";
    case GVOTE_ERR_WORKSPACE: return "workspace too small";
    case GVOTE_ERR_CAPACITY: return "size exceeds a supported maximum";
    case GVOTE_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}

int32_t gvote_abi_version(void) { return 1001; }

size_t gvote_workspace_bytes(const gvote_shape *shape, const gvote_item *items, int32_t n_items, int32_t S) {
  if (check_shape(shape) != GVOTE_OK || S < 1 || S > 128) return 0;
  if (check_items(shape, items, n_items, 0) != GVOTE_OK) return 0;
  return workspace_bytes_unchecked(shape, items, n_items, S);
}

gvote_status gvote_fit_gaussian(const gvote_shape *shape, const gvote_item *items, int32_t n_items, int32_t ddof,
                                float *mu, float *var, void *ws, size_t ws_bytes, void *stream) {
  gvote_status st = check_shape(shape);
  if (st != GVOTE_OK) return st;
  if ((st = check_items(shape, items, n_items, NEED_HIDDEN)) != GVOTE_OK) return st;
  if (!mu || !var || !ws || (ddof != 0 && ddof != 1)) return GVOTE_ERR_INVALID_ARG;
  if (!aligned16(mu) || !aligned16(var) || !aligned16(ws)) return GVOTE_ERR_SHAPE;
  const FitPlan fp = plan_fit(shape, items, n_items);
  if (fp.max_batch_chunks > kMaxFitChunks) return GVOTE_ERR_CAPACITY;    // > 2.6e8 tokens in 32 items
  if (ws_bytes < fp.ws_bytes) return GVOTE_ERR_WORKSPACE;
  return launch_fit(shape, items, n_items, ddof, mu, var, ws, reinterpret_cast<hipStream_t>(stream));
}

gvote_status gvote_sample_queries(const gvote_shape *shape, const gvote_item *items, int32_t n_items, int32_t S,
                                  const float *mu, const float *var, void *q_out, void *h_tilde_out, void *ws,
                                  size_t ws_bytes, void *stream) {
  gvote_status st = check_shape(shape);
  if (st != GVOTE_OK) return st;
  if ((st = check_items(shape, items, n_items, NEED_WQ)) != GVOTE_OK) return st;
  if (!mu || !var || !q_out || !ws || S < 1) return GVOTE_ERR_INVALID_ARG;
  if (S > 128) return GVOTE_ERR_CAPACITY;
  if (!aligned16(mu) || !aligned16(var) || !aligned16(q_out) || !aligned16(ws) ||
      (h_tilde_out && !aligned16(h_tilde_out)))
    return GVOTE_ERR_SHAPE;
  if (ws_bytes < plan_sample(shape, n_items, S).ws_bytes) return GVOTE_ERR_WORKSPACE;
  return launch_sample(shape, items, n_items, S, mu, var, q_out, h_tilde_out, ws,
                       reinterpret_cast<hipStream_t>(stream));
}

gvote_status gvote_score_select(const gvote_shape *shape, const gvote_item *items, int32_t n_items, int32_t S,
                                const void *q, float p, int32_t mode, const int32_t *k_per_row, uint32_t *rowmask,
                                float *row_max, float *row_sum, void *ws, size_t ws_bytes, void *stream) {
  gvote_status st = check_shape(shape);
  if (st != GVOTE_OK) return st;
  if ((st = check_items(shape, items, n_items, NEED_K)) != GVOTE_OK) return st;
  if (!q || !rowmask || S < 1) return GVOTE_ERR_INVALID_ARG;
  if (S > 128) return GVOTE_ERR_CAPACITY;
  if (mode == GVOTE_SELECT_TOPP) {
    if (!(p > 0.0f) || p > 1.0f) return GVOTE_ERR_INVALID_ARG;
  } else if (mode == GVOTE_SELECT_TOPK) {
    if (!k_per_row) return GVOTE_ERR_INVALID_ARG;
  } else {
    return GVOTE_ERR_INVALID_ARG;
  }
  if (!aligned16(q) || (ws && !aligned16(ws))) return GVOTE_ERR_SHAPE;
  const size_t need = plan_score(shape, items, n_items, S).ws_bytes;
  if (!ws || ws_bytes < need) return GVOTE_ERR_WORKSPACE;
  return launch_score_select(shape, items, n_items, S, q, p, mode, k_per_row, rowmask, row_max, row_sum, ws,
                             ws_bytes, reinterpret_cast<hipStream_t>(stream));
}

gvote_status gvote_union_compact(const gvote_shape *shape, const gvote_item *items, int32_t n_items, int32_t S,
                                 const uint32_t *rowmask, uint32_t *union_mask, int32_t *budget, int64_t *offsets,
                                 void *k_out, void *v_out, int32_t *idx_out, int64_t capacity_tokens,
                                 int32_t *overflow_flag, void *ws, size_t ws_bytes, void *stream) {
  gvote_status st = check_shape(shape);
  if (st != GVOTE_OK) return st;
  if ((st = check_items(shape, items, n_items, NEED_K | NEED_V)) != GVOTE_OK) return st;
  if (!rowmask || !union_mask || !budget || !offsets || !k_out || !v_out || !overflow_flag || !ws || S < 1 ||
      capacity_tokens < 0)
    return GVOTE_ERR_INVALID_ARG;
  if (S > 128) return GVOTE_ERR_CAPACITY;
  if (!aligned16(k_out) || !aligned16(v_out) || !aligned16(ws)) return GVOTE_ERR_SHAPE;
  if (ws_bytes < plan_union(shape, items, n_items).ws_bytes) return GVOTE_ERR_WORKSPACE;
  return launch_union_compact(shape, items, n_items, S, rowmask, union_mask, budget,
                              reinterpret_cast<long long *>(offsets), k_out, v_out, idx_out, capacity_tokens,
                              overflow_flag, ws, reinterpret_cast<hipStream_t>(stream));
}

gvote_status gvote_union_compact_static(const gvote_shape *shape, const gvote_item *items, int32_t n_items, int32_t S,
                                        const uint32_t *rowmask, uint32_t *union_mask, int32_t *budget,
                                        int64_t *offsets, void *k_out, void *v_out, int32_t *idx_out,
                                        int64_t capacity_tokens, int32_t *overflow_flag, void *stream) {
  gvote_status st = check_shape(shape);
  if (st != GVOTE_OK) return st;
  if ((st = check_items(shape, items, n_items, NEED_K | NEED_V)) != GVOTE_OK) return st;
  if (!rowmask || !union_mask || !budget || !offsets || !k_out || !v_out || !overflow_flag || S < 1 ||
      capacity_tokens < 0)
    return GVOTE_ERR_INVALID_ARG;
  if (S > 128) return GVOTE_ERR_CAPACITY;
  if (!aligned16(k_out) || !aligned16(v_out)) return GVOTE_ERR_SHAPE;
  if (plan_union(shape, items, n_items).ws_bytes > kStaticScratchBytes) return GVOTE_ERR_CAPACITY;
  void *scratch_ptr = nullptr;
  if ((st = static_scratch_of_current_device(&scratch_ptr)) != GVOTE_OK) return st;
  return launch_union_compact(shape, items, n_items, S, rowmask, union_mask, budget,
                              reinterpret_cast<long long *>(offsets), k_out, v_out, idx_out, capacity_tokens,
                              overflow_flag, scratch_ptr, reinterpret_cast<hipStream_t>(stream));
}

gvote_status gvote_count_rows(const gvote_shape *shape, const gvote_item *items, int32_t n_items, int32_t S,
                              const uint32_t *rowmask, int32_t repeat, int32_t *counts, void *stream) {
  gvote_status st = check_shape(shape);
  if (st != GVOTE_OK) return st;
  if ((st = check_items(shape, items, n_items, 0)) != GVOTE_OK) return st;
  if (!rowmask || !counts || S < 1 || repeat < 1) return GVOTE_ERR_INVALID_ARG;
  if (S > 128) return GVOTE_ERR_CAPACITY;
  return launch_count_rows(shape, items, n_items, S, rowmask, repeat, counts, reinterpret_cast<hipStream_t>(stream));
}

gvote_status gvote_decode_attention(const gvote_shape *shape, int32_t n_items, const void *q, const void *k_out,
                                    const void *v_out, const int64_t *offsets, void *out, float *lse, void *ws,
                                    size_t ws_bytes, void *stream) {
  gvote_status st = check_shape(shape);
  if (st != GVOTE_OK) return st;
  if (n_items < 1 || !q || !k_out || !v_out || !offsets || !out || !ws) return GVOTE_ERR_INVALID_ARG;
  if (!aligned16(q) || !aligned16(k_out) || !aligned16(v_out) || !aligned16(out) || !aligned16(ws)) return GVOTE_ERR_SHAPE;
  const int ppr = shape->head_dim * (int)elem_bytes(shape->dtype) / 16;
  if (ppr < 1 || ppr > 64 || (ppr & (ppr - 1))) return GVOTE_ERR_UNSUPPORTED;
  if (ws_bytes < decode_ws_bytes(shape, n_items)) return GVOTE_ERR_WORKSPACE;
  return launch_decode_attention(shape, n_items, q, k_out, v_out, reinterpret_cast<const long long *>(offsets), out,
                                 lse, ws, reinterpret_cast<hipStream_t>(stream));
}

size_t gvote_decode_workspace_bytes(const gvote_shape *shape, int32_t n_items) {
  if (check_shape(shape) != GVOTE_OK || n_items < 1) return 0;
  return decode_ws_bytes(shape, n_items);
}

gvote_status gvote_attention_overlap(const gvote_shape *shape, const gvote_item *items, int32_t n_items, int32_t S,
                                     const void *q_real, const uint32_t *rowmask, float *overlap, void *ws,
                                     size_t ws_bytes, void *stream) {
  gvote_status st = check_shape(shape);
  if (st != GVOTE_OK) return st;
  if ((st = check_items(shape, items, n_items, NEED_K)) != GVOTE_OK) return st;
  if (!q_real || !rowmask || !overlap || !ws || S < 1) return GVOTE_ERR_INVALID_ARG;
  if (S > 128) return GVOTE_ERR_CAPACITY;
  if (!aligned16(q_real) || !aligned16(ws)) return GVOTE_ERR_SHAPE;
  if (ws_bytes < overlap_ws_bytes(shape, items, n_items)) return GVOTE_ERR_WORKSPACE;
  return launch_attention_overlap(shape, items, n_items, S, q_real, rowmask, overlap, ws,
                                  reinterpret_cast<hipStream_t>(stream));
}

int32_t gvote_debug_set_spin_limit(int32_t polls) { return set_hist_spin_limit(polls); }

gvote_status gvote_philox_u32(uint64_t seed, uint64_t stream_id, int64_t n, uint32_t *out, void *stream) {
  if (n < 0 || (n > 0 && !out)) return GVOTE_ERR_INVALID_ARG;
  return launch_philox_u32(seed, stream_id, n, out, reinterpret_cast<hipStream_t>(stream));
}

}  // extern "C"
