// Shared declarations of the gfx950 GVote library: descriptor tables that travel to the
// kernels by value (no device-side descriptor memory, so a call never copies or allocates),
// storage-type helpers, and the per-stage launch plans used both to size the workspace and
// to launch.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "gvote.h"

namespace gvote {

constexpr size_t kLdsBytesPerCu = 160 * 1024;   // LDS of one gfx950 compute unit

// Items per launch batch.  Tables are kernel arguments (<= 4 KiB), larger calls are split.
constexpr int kMaxItems = 32;

// The item a launch-wide chunk number falls into: the last item whose first chunk (`chunk0`, counted from `base`)
// is not beyond it.  Items are in ascending chunk order; a bisection over the table in the kernel arguments.
template <typename Table>
__device__ __forceinline__ int item_of_chunk(const Table &tab, int chunk, int base) {
  int lo = 0, hi = tab.n_items - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (chunk >= tab.it[mid].chunk0 - base) lo = mid;
    else hi = mid - 1;
  }
  return lo;
}

typedef unsigned short bf16_t;   // storage only; arithmetic is fp32

__device__ __forceinline__ float bf16_to_f32(bf16_t v) { return __uint_as_float(((uint32_t)v) << 16); }

// round-to-nearest-even, the rounding a model's bf16 store applies (inputs here are finite)
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// 16-byte vector of the storage type, widened to fp32.
template <typename T> struct Vec16;
template <> struct Vec16<float> {
  static constexpr int N = 4;
  __device__ __forceinline__ static void load(const float *p, float (&o)[4]) {
    const float4 v = *reinterpret_cast<const float4 *>(p);
    o[0] = v.x; o[1] = v.y; o[2] = v.z; o[3] = v.w;
  }
};
template <> struct Vec16<bf16_t> {
  static constexpr int N = 8;
  __device__ __forceinline__ static void load(const bf16_t *p, float (&o)[8]) {
    const uint4 v = *reinterpret_cast<const uint4 *>(p);
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xFFFF0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xFFFF0000u);
    o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xFFFF0000u);
    o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xFFFF0000u);
  }
};

// 16 bytes that are read once and never again (the big input streams): a non-temporal load keeps them
// from displacing anything in the caches; measured +8 % on the hidden-state stream.
typedef unsigned int u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4_t load_stream16(const void *p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
}
template <typename T> struct Vec16Stream;
template <> struct Vec16Stream<float> {
  __device__ __forceinline__ static void load(const float *p, float (&o)[4]) {
    const u32x4_t v = load_stream16(p);
    o[0] = __uint_as_float(v.x); o[1] = __uint_as_float(v.y); o[2] = __uint_as_float(v.z); o[3] = __uint_as_float(v.w);
  }
};
template <> struct Vec16Stream<bf16_t> {
  __device__ __forceinline__ static void load(const bf16_t *p, float (&o)[8]) {
    const u32x4_t v = load_stream16(p);
    o[0] = __uint_as_float(v.x << 16); o[1] = __uint_as_float(v.x & 0xFFFF0000u);
    o[2] = __uint_as_float(v.y << 16); o[3] = __uint_as_float(v.y & 0xFFFF0000u);
    o[4] = __uint_as_float(v.z << 16); o[5] = __uint_as_float(v.z & 0xFFFF0000u);
    o[6] = __uint_as_float(v.w << 16); o[7] = __uint_as_float(v.w & 0xFFFF0000u);
  }
};

template <typename T> __device__ __forceinline__ float to_f32(T v);
template <> __device__ __forceinline__ float to_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f32<bf16_t>(bf16_t v) { return bf16_to_f32(v); }
template <typename T> __device__ __forceinline__ T from_f32(float v);
template <> __device__ __forceinline__ float from_f32<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f32<bf16_t>(float v) { return f32_to_bf16(v); }

// Accumulator of a dot product over stored values: fp32 for bf16 storage (products of bf16 are exact
// in fp32), fp64 for fp32 storage so that the fp32 configuration keeps its 1e-5 agreement.
template <typename T> struct Acc { typedef float type; };
template <> struct Acc<float> { typedef double type; };

// One step of the weighted most-significant-digit-first search, run by ONE wave (all 64 lanes):
// walking the 256 digit bins from 255 down, find the first non-empty digit at which `above` plus
// the weights met so far reaches `target`; if rounding leaves the total short, take the lowest
// non-empty digit.  Returns the digit; `above` becomes the weight strictly above it.
template <typename H>
__device__ __forceinline__ int pick_digit_wave(const H *hist, const int *cnt, double &above, double target,
                                               int lane) {
  // lane 0 holds digits 255..252, lane 63 digits 3..0
  double h[4];
  int c[4];
  double mine = 0.0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int dg = 255 - (lane * 4 + i);
    h[i] = (double)hist[dg];
    c[i] = cnt[dg];
    mine += h[i];
  }
  double x = mine;
  for (int off = 1; off < 64; off <<= 1) {
    const double y = __shfl_up(x, off, 64);
    if (lane >= off) x += y;
  }
  double cum = above + (x - mine);   // weight above this lane's first digit
  int pick = -1, low = -1;
  double cum_pick = 0.0, cum_low = 0.0;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int dg = 255 - (lane * 4 + i);
    if (c[i] != 0) {
      if (pick < 0 && cum + h[i] >= target) { pick = dg; cum_pick = cum; }
      low = dg;
      cum_low = cum;
    }
    cum += h[i];
  }
  const unsigned long long hit = __ballot(pick >= 0);
  int src;
  if (hit) {
    src = __ffsll((long long)hit) - 1;
  } else {
    const unsigned long long any = __ballot(low >= 0);
    src = 63 - __clzll((long long)any);
    pick = low;
    cum_pick = cum_low;
  }
  above = __shfl(cum_pick, src, 64);
  return __shfl(pick, src, 64);
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int ceil_div(int64_t a, int64_t b) { return (int)((a + b - 1) / b); }
inline size_t elem_bytes(int dtype) { return dtype == GVOTE_F32 ? 4 : 2; }

// ---------------------------------------------------------------- stage 1: fit
struct FitItem {
  const void *hidden;
  long long stride;     // elements
  int L, n_skip;
  int chunk0, n_chunks; // this item's row chunks are chunk0 .. chunk0 + n_chunks - 1
};
struct FitTable {
  int n_items, d, rows_per_chunk, pad;
  float *partial;       // [total_chunks][2][d]: chunk mean, chunk M2
  FitItem it[kMaxItems];
};
constexpr int kMaxFitChunks = 65535;   // row chunks of one launch batch (grid dimension y)
struct FitPlan {
  int rows_per_chunk;
  int total_chunks;            // over the whole call
  long long max_batch_chunks;  // most row chunks of any launch batch of the call
  size_t ws_bytes;
};
FitPlan plan_fit(const gvote_shape *sh, const gvote_item *items, int n_items);
gvote_status launch_fit(const gvote_shape *sh, const gvote_item *items, int n_items, int ddof, float *mu,
                        float *var, void *ws, hipStream_t st);

// ---------------------------------------------------------------- stage 2: sample + project + rotate
struct SampleItem {
  const void *w_q;
  const void *b_q;
  unsigned long long seed, stream_id;
  int pos0, n_future;
};
struct SampleTable {
  int n_items, d, S, SP;          // SP: samples padded to a multiple of 32 (MFMA blocks)
  int SPs, pad1;                  // SPs: samples padded to a multiple of 8: row pitch of the partial sums
  int n_out, head_dim, ksplits, kslice;
  float theta;
  int item0;                      // index of the batch's first item in the call (output offsets)
  const float *mu, *var;          // [n_items_call, d]
  void *h_tilde;                  // ws: [n_items_batch][S][d] storage type
  void *h_tilde_out;              // optional user copy, call-indexed
  float *partial;                 // ws: [n_items_batch][ksplits][n_out][SP]
  void *q_out;                    // [n_items_call][S][n_out]
  // the projection runs once per GROUP of consecutive items that share one W_q (requests through the same
  // layer): their samples are the columns of one product, W_q is read once per group
  int n_groups;
  unsigned char grp_first[kMaxItems], grp_count[kMaxItems];
  SampleItem it[kMaxItems];
};
struct SamplePlan {
  int SP, SPs, ksplits, kslice;
  size_t h_bytes_per_item, partial_bytes_per_item, ws_bytes;
};
SamplePlan plan_sample(const gvote_shape *sh, int n_items, int S);
gvote_status launch_sample(const gvote_shape *sh, const gvote_item *items, int n_items, int S, const float *mu,
                           const float *var, void *q_out, void *h_tilde_out, void *ws, hipStream_t st);
gvote_status launch_philox_u32(uint64_t seed, uint64_t stream_id, int64_t n, uint32_t *out, hipStream_t st);

// ---------------------------------------------------------------- stage 3: score + select
struct ScoreItem {
  const void *k;
  long long tok_stride, head_stride;   // elements
  long long mask_off;                  // first word of this item's rowmask block
  int L, W;                            // W = words per row
  int row0;                            // first global row of this item within the batch
  int pad;
};
struct ScoreTable {
  int n_items, S, n_q_heads, n_kv_heads;
  int head_dim, mode, rows_per_item, item0;
  float p, pad2;
  double scale;                        // 1 / sqrt(head_dim)
  const void *q;                       // [n_items_call][S][H_q][d_k]
  const int *k_per_row;                // call-indexed or null
  uint32_t *rowmask;
  float *row_max, *row_sum;            // call-indexed or null
  const int *row_list;                 // null (every row of the batch), or the batch rows to process ...
  const int *n_list;                   // ... and how many there are (device side)
  int *n_fallback;                     // null, or counter incremented once per row this kernel processes
  float *lg_cache;                     // null, or cache_rows slices of cache_stride floats (one per workgroup)
  long long cache_stride;
  int cache_rows, pad5;
  ScoreItem it[kMaxItems];
};
struct ScorePlan { size_t ws_bytes; };

// bf16 fast path (score_fast.hip)
constexpr int kBins = 256;            // histogram bins per row: 16 units of logit below the window top (the top sits up to 4 units above the maximum)
constexpr int kBinsPerUnit = 16;      // bins per unit of logit: bin width 1/16, window 16 units
constexpr int kCandCap = 4096;        // boundary-bin candidates a row may collect before it is redone exactly
constexpr int kSubCap = 16;           // entries of one candidate sub-list (row, key chunk, wave, lane half)
constexpr int kOvfCap = 256;          // entries of a row's shared overflow list (for sub-lists that fill up)
struct RowInfo {
  float mdot;       // row maximum of the raw dot product
  int astar;        // absolute bin index floor(dot * c1) in which the cut falls
  int flag;         // odd: redo this row with the general selector (1 window, 3 lists full, 5 too many candidates, 7 pass 1 gave up); 2: second resolve tier;
                    // 4 (between find_bin and refine_bin only): too many keys in the cut bin, look inside it with finer bins
  int shift;        // astar counts bins of 2^-shift standard bins (0; 8 once the cut bin has been looked into)
  double above;     // weight of all keys in bins above astar (relative to exp(-max)); their number in TOPK mode
  double target;    // p * Z; k in TOPK mode
};
struct FastItem {
  const void *k;
  long long tok_stride, head_stride;
  long long mask_off;
  long long tmax0;  // first entry of the item's [H_kv][W][NQ] tile bins
  int L, W;
  int n_chunks;     // key chunks per KV head
  int wg0;          // first workgroup of the item
  int part0;        // first (head, chunk) slot of the item in the partial arrays
  int pad;
};
struct FastTable {
  int n_items, S, Hq, Hkv, G, NQ, NQB, chunk_keys;
  int item0, rows_per_item;
  int n_slots;              // (item, KV head, chunk) slots of the batch
  int emit_split;           // pass 2 cuts every chunk into this many pieces of at most 8192 keys (its LDS mask buffer)
  int mode;                 // gvote_select_mode: TOPP bins softmax weights, TOPK bins key counts
  int sub_per_row;          // candidate sub-lists per row = 16 * (most key chunks of an item in the batch)
  int spin_limit;           // polls a finished pass-1 wave waits for the others before it gives up
  float scale, c1, c2, p;   // c1 = bins per raw-dot unit, c2 = log2(e) / sqrt(d_k)
  const void *q;
  const int *k_per_row;     // TOPK: call-indexed row budgets
  uint32_t *rowmask;
  float *row_max, *row_sum;
  float *part_max;          // [slot][NQ]: chunk maximum of the raw dot
  int *part_top;            // [slot][NQ]: top (absolute bin) of the chunk's histogram window
  uint32_t *part_hist;      // [slot][NQ][kBins]: fixed-point bin weights; last bin: a float's bits
  short *tile_bin;          // per (item, KV head, 32-key tile, row): bin of the largest raw dot, written by pass 1
  RowInfo *info;            // [rows of the batch]
  int *n_fallback;          // counter of rows redone by the general selector (first word of the workspace)
  int *n_list;              // rows of this batch waiting for the general selector (second word) ...
  int *n_refine;            // words 8..: rows whose cut lies below their window, per refinement level (device-side early exits)
  int *row_list;            // ... and their batch row indices
  int *cand_cnt;            // [rows][sub_per_row]: entries in each sub-list
  uint2 *cands;             // [rows][sub_per_row][kSubCap]: (raw dot bits, position)
  int *ovf_cnt;             // [rows]: entries in the row's overflow list
  uint2 *ovf;               // [rows][kOvfCap]
  FastItem it[kMaxItems];
};
struct FastPlan { size_t off_max, off_top, off_hist, off_info, off_cnt, off_cands, off_tmax, off_list, off_ovfc, off_ovf, ws_bytes; };
bool fast_path_ok(const gvote_shape *sh, int S, int mode, float p);
int set_hist_spin_limit(int polls);   // returns the previous limit; negative restores the default
FastPlan plan_fast(const gvote_shape *sh, const gvote_item *items, int n_items, int S);
gvote_status launch_score_fast(const gvote_shape *sh, const gvote_item *items, int n_items, int S, const void *q,
                               float p, int mode, const int *k_per_row, uint32_t *rowmask, float *row_max,
                               float *row_sum, void *ws, hipStream_t st);
// the exact general selector on a batch of <= kMaxItems items; with `row_list` only the listed rows
gvote_status launch_select_rows_general(const gvote_shape *sh, const gvote_item *items, int nb, int item0, int S,
                                        const void *q, float p, int mode, const int *k_per_row, uint32_t *rowmask,
                                        long long mask_off0, float *row_max, float *row_sum, const int *row_list,
                                        const int *n_list, int *n_fallback, float *lg_cache, size_t cache_bytes,
                                        hipStream_t st);
size_t general_cache_bytes(const gvote_item *items, int n_items);
ScorePlan plan_score(const gvote_shape *sh, const gvote_item *items, int n_items, int S);
gvote_status launch_score_select(const gvote_shape *sh, const gvote_item *items, int n_items, int S, const void *q,
                                 float p, int mode, const int *k_per_row, uint32_t *rowmask, float *row_max,
                                 float *row_sum, void *ws, size_t ws_bytes, hipStream_t st);

// ---------------------------------------------------------------- stage 4: union + count + compact
constexpr int kChunkWords = 64;        // a compaction chunk = 64 mask words = 2048 tokens
struct UnionItem {
  const void *k, *v;
  long long tok_stride, head_stride;
  long long rowmask_off, union_off;    // first word of the item's blocks
  int L, W;
  int n_chunks;                        // chunks per KV head = ceil(W / kChunkWords)
  int chunk0;                          // global id of (item, head 0, chunk 0)
};
struct UnionTable {
  int n_items, S, n_q_heads, n_kv_heads;
  int head_dim, item0, total_chunks_call, n_heads_call;
  const uint32_t *rowmask;
  uint32_t *union_mask;
  int *chunk_count;                    // ws [total_chunks_call]
  long long *chunk_base;               // ws [total_chunks_call + 1]
  int *head_first;                     // ws [n_heads_call + 1]: first chunk of each (item, head)
  void *k_out, *v_out;
  int *idx_out;
  long long capacity;
  UnionItem it[kMaxItems];
};
struct UnionPlan { int total_chunks; size_t off_base, off_head, ws_bytes; };
UnionPlan plan_union(const gvote_shape *sh, const gvote_item *items, int n_items);
// the static scratch array of stage 4 (one per device): its size, and its address on the current device
constexpr size_t kStaticScratchBytes = 1 << 20;
gvote_status static_scratch_of_current_device(void **ptr);
gvote_status launch_union_compact(const gvote_shape *sh, const gvote_item *items, int n_items, int S,
                                  const uint32_t *rowmask, uint32_t *union_mask, int *budget, long long *offsets,
                                  void *k_out, void *v_out, int *idx_out, long long capacity, int *overflow_flag,
                                  void *ws, hipStream_t st);

gvote_status launch_count_rows(const gvote_shape *sh, const gvote_item *items, int n_items, int S,
                               const uint32_t *rowmask, int repeat, int *counts, hipStream_t st);

size_t overlap_ws_bytes(const gvote_shape *sh, const gvote_item *items, int n_items);
size_t decode_ws_bytes(const gvote_shape *sh, int n_items);
gvote_status launch_decode_attention(const gvote_shape *sh, int n_items, const void *q, const void *k_out,
                                     const void *v_out, const long long *offsets, void *out, float *lse, void *ws,
                                     hipStream_t st);
gvote_status launch_attention_overlap(const gvote_shape *sh, const gvote_item *items, int n_items, int S,
                                      const void *q_real, const uint32_t *rowmask, float *overlap, void *ws,
                                      hipStream_t st);

#define GVOTE_CHECK_LAUNCH()                                  \
  do {                                                        \
    if (hipGetLastError() != hipSuccess) return GVOTE_ERR_HIP; \
  } while (0)

}  // namespace gvote
