/*
 * gvote.h - C ABI of the MI355X (gfx950) implementation of GVote's budget-free
 * KV-cache selection: the per-request, per-layer procedure of the paper's Sec. 3.2
 * (Steps 2-4) and Algorithm 1, with the per-query selection rule of Sec. 3.1
 * (the smallest key set whose softmax mass reaches p).
 *
 * One "item" is one (request, layer) pair; every call processes n_items items in one
 * batch of launches on the caller's HIP stream.  The four calls are the four stages:
 *
 *   gvote_fit_gaussian    Step 2: per-channel mean / variance of the prefill hidden states
 *   gvote_sample_queries  Step 3: draw S hidden states, project with W_q, rotate (RoPE)
 *   gvote_score_select    Eq. (1) logits of every synthetic query against every cached key,
 *                         then the Sec. 3.1 top-p set of each query row, as bit masks
 *   gvote_union_compact   Step 4: OR the row masks of a KV group into the keep-set, count it
 *                         (the adaptive budget B), gather the kept K/V rows
 *
 * Conventions
 *   - All data pointers are DEVICE pointers unless a parameter says "host".  gvote_shape and
 *     the gvote_item array are HOST memory and are only read during the call.
 *   - The caller owns every buffer, including the workspace `ws` whose minimum size
 *     gvote_workspace_bytes() returns.  The library allocates, frees and retains nothing.
 *   - `stream` is a hipStream_t (NULL = the default stream).  Calls only enqueue work: they
 *     never synchronise, so outputs are valid once the stream has reached that point.
 *     Calls that share a workspace must be issued on one stream (or otherwise ordered).
 *     No call allocates, copies, clears memory through the runtime or waits: a caller may record
 *     the calls into a HIP graph and replay it.
 *   - Errors are returned as gvote_status.  Everything that can be checked on the host (null
 *     pointers, shapes, alignment, workspace size, unsupported types) is rejected before any
 *     launch, leaving all outputs untouched.  A failing HIP launch gives GVOTE_ERR_HIP.
 *   - Alignment: every data pointer is 16-byte aligned; d_model, head_dim, hidden_row_stride,
 *     kv_tok_stride and kv_head_stride are multiples of 8 elements.  The innermost dimension of
 *     every tensor is contiguous.
 *   - Row order: query row r = s * n_q_heads + h (sample-major); query head h belongs to KV
 *     head h / G with G = n_q_heads / n_kv_heads.
 *   - Bit masks: key t of a row is bit (t % 32) of 32-bit word t / 32; a row of an item with
 *     context length L has W = (L + 31) / 32 words; bits at positions >= L are 0.
 */
#ifndef GVOTE_H
#define GVOTE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define GVOTE_API __attribute__((visibility("default")))

typedef enum {
  GVOTE_OK = 0,
  GVOTE_ERR_INVALID_ARG = 1,  /* null pointer, n_items < 1, S < 1, p outside (0, 1], ddof not 0/1 ... */
  GVOTE_ERR_SHAPE = 2,        /* inconsistent or misaligned shape / stride / pointer */
  GVOTE_ERR_UNSUPPORTED = 3,  /* valid request this build has no kernel for */
  GVOTE_ERR_WORKSPACE = 4,    /* ws_bytes < gvote_workspace_bytes(...) */
  GVOTE_ERR_CAPACITY = 5,     /* a size exceeds a stated maximum */
  GVOTE_ERR_HIP = 6           /* a HIP runtime call or launch failed */
} gvote_status;

typedef enum { GVOTE_F32 = 0, GVOTE_BF16 = 1 } gvote_dtype;

/* How each synthetic query row picks its keys.
 * TOPP: Sec. 3.1 "required keys": shortest prefix, in the order (logit descending, position
 *       ascending), whose un-normalised softmax weight reaches p * Z.
 * TOPK: Algorithm 1's row-wise TopK on logits with a caller-given k per row (same order). */
typedef enum { GVOTE_SELECT_TOPP = 0, GVOTE_SELECT_TOPK = 1 } gvote_select_mode;

/* Model geometry shared by all items of a call.
 * d_model % 8 == 0; n_q_heads % n_kv_heads == 0; head_dim % 8 == 0, 8 <= head_dim <= 256.
 * dtype is the storage type of hidden, w_q, b_q, k, v, q and k_out / v_out; statistics,
 * logits and softmax weights are always fp32.
 * RoPE: frequencies rope_theta^(-2i/head_dim), pairing (i, i + head_dim/2) ("rotate half"). */
typedef struct {
  int32_t d_model;
  int32_t n_q_heads;
  int32_t n_kv_heads;
  int32_t head_dim;
  int32_t dtype;      /* gvote_dtype */
  float rope_theta;
} gvote_shape;

/* One (request, layer).  Strides are in ELEMENTS.
 * hidden  [L, d_model]: the layer's normalised input (what W_q multiplies), row t at t * hidden_row_stride.
 * w_q     [n_q_heads * head_dim, d_model] row-major (linear-layer layout: out x in), dense.
 * b_q     [n_q_heads * head_dim] or NULL.
 * k, v    element (t, h, c) at t * kv_tok_stride + h * kv_head_stride + c; keys are cached
 *         post-RoPE, as a KV cache holds them.
 * L       context length, >= 2.  n_skip: leading tokens left out of the fit (the paper's n_s), 0 <= n_skip <= L - 2.
 * pos0, n_future: the synthetic queries are rotated with cos / sin averaged over positions
 *         pos0 .. pos0 + n_future - 1 (Alg. 1 "AverageCosSin(n_f)"); the next decode position
 *         alone is pos0 = L, n_future = 1.  1 <= n_future <= 4096.
 * seed, stream_id: Philox4x32-10 key and upper counter words of this item's draws. */
typedef struct {
  const void *hidden;
  int64_t hidden_row_stride;
  const void *w_q;
  const void *b_q;
  const void *k;
  const void *v;
  int64_t kv_tok_stride;
  int64_t kv_head_stride;
  int32_t L;
  int32_t n_skip;
  int32_t pos0;
  int32_t n_future;
  uint64_t seed;
  uint64_t stream_id;
} gvote_item;

/* Static text for a status code (never NULL). */
GVOTE_API const char *gvote_status_string(gvote_status st);

/* Library ABI version (major * 1000 + minor). */
GVOTE_API int32_t gvote_abi_version(void);

/* Bytes of device workspace that any of the four calls may need for this batch (the maximum
 * over the calls, so one buffer serves all four).  Returns 0 if the arguments are invalid. */
GVOTE_API size_t gvote_workspace_bytes(const gvote_shape *shape, const gvote_item *items, int32_t n_items, int32_t S);

/* Step 2 (Sec. 3.2; Alg. 1 "mu <- mean(h), sigma^2 <- var(h)").
 * mu[i, j], var[i, j] (fp32, [n_items, d_model]) = mean and variance over tokens
 * n_skip .. L-1 of hidden[:, j]; var divides by (n - ddof), ddof in {0, 1}.
 * Reads items[].hidden / hidden_row_stride / L / n_skip. */
GVOTE_API gvote_status gvote_fit_gaussian(const gvote_shape *shape, const gvote_item *items, int32_t n_items,
                                int32_t ddof, float *mu, float *var,
                                void *ws, size_t ws_bytes, void *stream);

/* Step 3 (Sec. 3.2; Alg. 1 "H~ ~ N(mu, diag sigma^2)", "AverageCosSin(n_f)", "Q~ = RoPE(H~ W_q, P)").
 * For item i and sample s: z[s, j] is the Box-Muller normal of Philox draw s * d_model + j
 * (block = draw >> 2 in counter words 0..1, stream_id in words 2..3, key = seed; u =
 * ((x >> 9) + 0.5) * 2^-23; words (0,1) and (2,3) pair up, even word -> r cos, odd -> r sin);
 * h~ = mu + sqrt(var) * z rounded to dtype; q = h~ W_q^T + b_q accumulated in fp32; RoPE; rounded
 * to dtype into q_out[i, s, h, c] ([n_items, S, n_q_heads, head_dim]).
 * h_tilde_out ([n_items, S, d_model], dtype) is optional (NULL to skip): the sampled hidden states.
 * 1 <= S <= 128. */
GVOTE_API gvote_status gvote_sample_queries(const gvote_shape *shape, const gvote_item *items, int32_t n_items,
                                  int32_t S, const float *mu, const float *var,
                                  void *q_out, void *h_tilde_out,
                                  void *ws, size_t ws_bytes, void *stream);

/* Eq. (1) logits + Sec. 3.1 selection.  For every row r = (s, h) of every item:
 * l_t = <q[i, s, h, :], k[t, h / G, :]> / sqrt(head_dim) over all L keys (no causal mask: the
 * queries lie in the future), m = max l, w_t = exp(l_t - m), Z = sum w; the row's set is chosen by
 * `mode` (TOPP uses p in (0, 1]; p >= 1 keeps every key; TOPK uses k_per_row[n_items * S * n_q_heads],
 * device int32, clamped to [1, L]; pass NULL for TOPP).  Ties are broken towards the lower position.
 * rowmask: items back to back, item i holding [S * n_q_heads, W_i] words.
 * row_max, row_sum: optional [n_items, S * n_q_heads] fp32 diagnostics (m and Z), NULL to skip.
 * ws is required (gvote_workspace_bytes): statistics between the passes and the exact selector's logit cache.
 * Range: on the matrix-core path logits beyond +-65536 (after the 1/sqrt(head_dim) scaling) are treated as +-65536
 * by the histogram search; infinities and NaN in q or K never cause an invalid access, the affected rows' results are
 * unspecified.
 * Diagnostics: when the matrix-core path runs (bf16, head_dim 64 or 128, every L >= 32; TOPP with p < 1, or TOPK) the first int32
 * words of ws hold, after the call and until ws is used again: [0] the number of rows that had to be redone by
 * the exact general selector, and [2..5] that number by reason: the cut lies below the histogram windows (two
 * windows of 16 logit units each, the first starting up to 4 units above the row maximum); a row's candidate lists
 * are full; more candidates around the cut than the resolver holds; a first-pass workgroup gave up waiting for
 * one of its waves (see gvote_debug_set_spin_limit) - such rows are never answered from a partial histogram;
 * [6] the number of rows whose cut lay below the first window and was found in the second (those
 * rows cost one more pass over K for their block of 64 rows, not the exact selector). */
GVOTE_API gvote_status gvote_score_select(const gvote_shape *shape, const gvote_item *items, int32_t n_items,
                                int32_t S, const void *q, float p, int32_t mode, const int32_t *k_per_row,
                                uint32_t *rowmask, float *row_max, float *row_sum,
                                void *ws, size_t ws_bytes, void *stream);

/* Step 4 (Sec. 3.2; Alg. 1 "K <- union of C^(s)", "prune (K, V) to the indices in K"; Sec. 3.4:
 * masks, one OR, nonzero, gather).
 * union_mask: items back to back, item i holding [n_kv_heads, W_i] words: OR of the S * G row masks
 *             of each KV head.
 * budget[i, h] (int32) = popcount of that head's union = the adaptive budget B.
 * offsets[n_items * n_kv_heads + 1] (int64): exclusive prefix sum of budget in (item, head) order.
 * k_out, v_out [capacity_tokens, head_dim] (dtype): head (i, h) owns rows offsets[.] .. offsets[.+1]-1,
 *             its kept tokens in ascending position, copied bit for bit.
 * idx_out [capacity_tokens] (int32, optional): the positions t of those rows.
 * Rows at or beyond capacity_tokens are not written and *overflow_flag (device int32) is set to 1,
 * otherwise to 0; budget and offsets are always complete.  capacity_tokens = sum_i L_i * n_kv_heads
 * can never overflow. */
GVOTE_API gvote_status gvote_union_compact(const gvote_shape *shape, const gvote_item *items, int32_t n_items,
                                 int32_t S, const uint32_t *rowmask,
                                 uint32_t *union_mask, int32_t *budget, int64_t *offsets,
                                 void *k_out, void *v_out, int32_t *idx_out,
                                 int64_t capacity_tokens, int32_t *overflow_flag,
                                 void *ws, size_t ws_bytes, void *stream);

/* gvote_union_compact for callers that cannot allocate device memory or carry a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as
 * gvote_union_compact without `ws`: the chunk counts, chunk bases and head indices of the call live in a
 * fixed 1 MiB array inside the library's device image (one copy per GPU, held until the process ends).
 * The call allocates and frees nothing.  Limit: 12 bytes per 2048-token chunk of a KV head plus 4 per
 * (item, head) must fit the array (about 87 000 chunks, i.e. 1.7e8 head-tokens per call); larger calls
 * return GVOTE_ERR_CAPACITY before any launch.  The calling thread's current device must be the stream's
 * device; the array's address is looked up on the first call on each device.  All calls on one GPU share
 * the array (every call rewrites all of it that it reads, nothing needs clearing): calls that overlap in
 * time on one GPU race - issue them on one stream or order them. */
GVOTE_API gvote_status gvote_union_compact_static(const gvote_shape *shape, const gvote_item *items, int32_t n_items,
                                 int32_t S, const uint32_t *rowmask,
                                 uint32_t *union_mask, int32_t *budget, int64_t *offsets,
                                 void *k_out, void *v_out, int32_t *idx_out,
                                 int64_t capacity_tokens, int32_t *overflow_flag, void *stream);

/* Alg. 1 "B_step <- |C_0|": sizes of row sets.  counts[i, c, r] (device int32, [n_items, repeat, S * n_q_heads])
 * = number of keys selected in row r of item i's row masks, written `repeat` times over.  With the masks
 * of the REAL current query (S = 1, GVOTE_SELECT_TOPP) and repeat = number of synthetic samples, the
 * output is exactly the k_per_row that GVOTE_SELECT_TOPK expects for the synthetic rows (row s * n_q_heads
 * + h gets the budget of head h): Alg. 1's row-wise TopK with the real query's budget.  repeat >= 1. */
GVOTE_API gvote_status gvote_count_rows(const gvote_shape *shape, const gvote_item *items, int32_t n_items, int32_t S,
                                        const uint32_t *rowmask, int32_t repeat, int32_t *counts, void *stream);

/* Consumer of the compressed cache (Sec. 3.4: a non-uniform per-head cache behind a variable-length
 * attention interface; Eq. (1)-(2)).  One decode query per item and head: q[n_items, n_q_heads, head_dim]
 * (dtype); head h of item i attends to rows offsets[i*n_kv_heads + h/G] .. offsets[.. + 1] - 1 of the packed
 * k_out / v_out that gvote_union_compact produced:  out[i, h, :] = softmax(q K^T / sqrt(head_dim)) V, rounded
 * to dtype ([n_items, n_q_heads, head_dim]); lse[i, h] (fp32, optional) = log sum exp of the logits.
 * head_dim * element size / 16 must be a power of two <= 64 (else GVOTE_ERR_UNSUPPORTED).
 * ws: gvote_decode_workspace_bytes(shape, n_items) bytes (also covered by gvote_workspace_bytes for the same
 * n_items): the packed rows of a head are shared out over several workgroups whose partial results meet there. */
GVOTE_API gvote_status gvote_decode_attention(const gvote_shape *shape, int32_t n_items, const void *q,
                                              const void *k_out, const void *v_out, const int64_t *offsets,
                                              void *out, float *lse, void *ws, size_t ws_bytes, void *stream);
GVOTE_API size_t gvote_decode_workspace_bytes(const gvote_shape *shape, int32_t n_items);

/* Sec. 3.3 "Attention Overlap": overlap[i, s, h] (fp32, [n_items, S, n_q_heads]) = the share of the REAL query
 * q_real[i, h, :]'s attention (softmax over all L keys of KV head h/G) that falls on the keys selected in row
 * (s, h) of rowmask.  q_real [n_items, n_q_heads, head_dim] (dtype).  ws: gvote_workspace_bytes. */
GVOTE_API gvote_status gvote_attention_overlap(const gvote_shape *shape, const gvote_item *items, int32_t n_items,
                                               int32_t S, const void *q_real, const uint32_t *rowmask,
                                               float *overlap, void *ws, size_t ws_bytes, void *stream);

/* Test aid for the failure handling of gvote_score_select's first pass: a wave that has finished its keys
 * polls for the other waves of its workgroup at most `polls` times before it gives up and the workgroup's
 * rows go to the exact selector (default 1 << 22, never reached in normal operation; 0 makes nearly every
 * workgroup give up, so the error path can be tested while every kernel still exits normally).  Process-wide,
 * applies to later calls; a negative value restores the default.  Returns the previous limit. */
GVOTE_API int32_t gvote_debug_set_spin_limit(int32_t polls);

/* Test aid: out[e] (device uint32, e < n) = Philox4x32-10 draw e of stream (seed, stream_id),
 * the integer stream gvote_sample_queries consumes. */
GVOTE_API gvote_status gvote_philox_u32(uint64_t seed, uint64_t stream_id, int64_t n, uint32_t *out, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* GVOTE_H */
