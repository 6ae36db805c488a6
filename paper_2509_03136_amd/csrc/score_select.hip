// Stage 3 - scores and per-query selection (paper Eq. (1): logits Q~ K^T / sqrt(d_k) and their
// softmax; Sec. 3.1: a query's required keys are the smallest set whose attention mass reaches
// p; Alg. 1's row-wise TopK on logits is the same search with unit weights).
//
// select_row_kernel: the exact, general selector.  One workgroup owns one query row (s, h) and
// recomputes its logits from K in every pass, so nothing of size S*H_q*L is ever stored.
//   pass 0      m = max_t l_t
//   pass 1..4   most-significant-digit-first radix search, 8 bits per pass, over the
//               order-preserving 32-bit image of the fp32 logit.  Each pass histograms the
//               WEIGHT exp(l - m) (or 1 for TopK) of the keys that still match the digits found
//               so far; walking the 256 bins from the top finds the digit where the cumulative
//               weight crosses p*Z (or k).  After four passes the threshold logit tau is known
//               exactly, with the weight strictly above it and the number of keys equal to it.
//   pass 5      emit bits: l > tau, plus the first n ties in position order, n the least count
//               that reaches the target (ties are broken towards the lower position).
// The logit of a key is computed by the same instruction sequence in every pass, so passes agree
// bit for bit.
#include <algorithm>

#include "gvote_internal.hpp"

namespace gvote {

namespace {

constexpr int kSelThreads = 1024;

// fp32 -> uint32 that sorts like the float
__device__ __forceinline__ uint32_t ordered_bits(float f) {
  const uint32_t b = __float_as_uint(f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float from_ordered_bits(uint32_t u) {
  return __uint_as_float((u & 0x80000000u) ? (u ^ 0x80000000u) : ~u);
}

// weights in 2^-40 units of the row maximum's weight (integer LDS atomics; float ones run ~30x slower)
constexpr double kSelFix = 1099511627776.0;

template <typename T>
__device__ __forceinline__ void select_row_body(const ScoreTable &tab, int grow, float *cache) {
  // `cache` (null or L floats of workspace owned by this workgroup): the row's logits, written by pass 0
  // and re-read by the later passes instead of recomputing them; a thread only re-reads what it wrote.
  constexpr int NV = Vec16<T>::N;
  constexpr int NW = kSelThreads / 64;
  const int it = grow / tab.rows_per_item;
  const int r = grow - it * tab.rows_per_item;
  const int s = r / tab.n_q_heads, h = r - s * tab.n_q_heads;
  const int kvh = h / (tab.n_q_heads / tab.n_kv_heads);
  const ScoreItem I = tab.it[it];
  const int dk = tab.head_dim;
  const int L = I.L;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const bool topk = tab.mode == GVOTE_SELECT_TOPK;

  __shared__ float q_s[256];
  __shared__ float lg[kSelThreads];          // logits of the current tile of kSelThreads keys
  __shared__ unsigned long long hist[256];
  __shared__ int cnt[256];
  __shared__ float red_f[NW];
  __shared__ int red_i[NW];
  __shared__ uint32_t sh_prefix;
  __shared__ double sh_above, sh_target, sh_z;
  __shared__ int sh_ties, sh_take, sh_tie_base;

  const T *qrow = reinterpret_cast<const T *>(tab.q) + ((size_t)(tab.item0 + it) * tab.rows_per_item + r) * dk;
  if (tid < dk) q_s[tid] = to_f32<T>(qrow[tid]);
  if (tid == 0) {
    sh_prefix = 0u;
    sh_above = 0.0;
    if (tab.n_fallback) atomicAdd(tab.n_fallback, 1);
  }
  __syncthreads();

  const T *kbase = reinterpret_cast<const T *>(I.k) + (long long)kvh * I.head_stride;
  typedef typename Acc<T>::type acc_t;
  const acc_t scale = (acc_t)tab.scale;
  // A key row is read by `lpk` neighbouring lanes, 16 bytes each (coalesced), the partial dot products
  // are added across those lanes; every pass forms a key's logit by this very sequence.
  const int ppr = dk / NV;                    // 16-byte pieces of a key row
  int lpk = 1;
  while (lpk < ppr) lpk <<= 1;                // lanes per key: power of two, <= 32
  const int kpi = kSelThreads / lpk;          // keys per sweep of the workgroup
  const int slot = tid / lpk, piece = tid - slot * lpk;
  auto fill_tile = [&](int tile0) {           // lg[i] = logit of key tile0 + i, i < kSelThreads
    constexpr int UN = 8;                     // key rows in flight per lane
    for (int k0 = 0; k0 < kSelThreads; k0 += UN * kpi) {
      float kv[UN][NV];
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        const int t = tile0 + k0 + u * kpi + slot;
        const int tc = t < L ? t : L - 1;     // in bounds; the result is dropped below
        Vec16<T>::load(kbase + (long long)tc * I.tok_stride + (piece < ppr ? piece : 0) * NV, kv[u]);
      }
#pragma unroll
      for (int u = 0; u < UN; ++u) {
        if (k0 + u * kpi < kSelThreads) {     // (only matters when a sweep covers more than 1/8 of the tile)
          acc_t acc = 0;
          if (piece < ppr) {
#pragma unroll
            for (int i = 0; i < NV; ++i) acc = fma((acc_t)q_s[piece * NV + i], (acc_t)kv[u][i], acc);
          }
          for (int off = lpk >> 1; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
          if (piece == 0) lg[k0 + u * kpi + slot] = (float)(acc * scale) + 0.0f;   // "+ 0": -0 becomes +0
        }
      }
    }
  };

  // ---- pass 0: row maximum
  float m = -INFINITY;
  for (int tile0 = 0; tile0 < L; tile0 += kSelThreads) {
    fill_tile(tile0);
    __syncthreads();
    if (tile0 + tid < L) {
      m = fmaxf(m, lg[tid]);
      if (cache) cache[tile0 + tid] = lg[tid];
    }
    __syncthreads();
  }
  for (int off = 32; off > 0; off >>= 1) m = fmaxf(m, __shfl_xor(m, off, 64));
  if (lane == 0) red_f[wave] = m;
  __syncthreads();
  m = red_f[0];
  for (int w = 1; w < NW; ++w) m = fmaxf(m, red_f[w]);
  __syncthreads();

  const bool keep_all = !topk && tab.p >= 1.0f;
  const int n_pass = keep_all ? 1 : 4;
  auto fixed_weight = [&](float l) -> unsigned long long {
    return topk ? 1ull : (unsigned long long)((double)expf(l - m) * kSelFix);
  };

  // ---- passes 1..4: weighted radix search for the threshold
  for (int pass = 0; pass < n_pass; ++pass) {
    const int shift = 24 - 8 * pass;
    if (tid < 256) { hist[tid] = 0ull; cnt[tid] = 0; }
    __syncthreads();
    const uint32_t prefix = sh_prefix;
    for (int tile0 = 0; tile0 < L; tile0 += kSelThreads) {
      if (!cache) {
        fill_tile(tile0);
        __syncthreads();
      }
      if (tile0 + tid < L) {
        const float l = cache ? cache[tile0 + tid] : lg[tid];
        const uint32_t u = ordered_bits(l);
        if (pass == 0 || (u >> (shift + 8)) == prefix) {
          const int dg = (u >> shift) & 255;
          atomicAdd(&hist[dg], fixed_weight(l));
          atomicAdd(&cnt[dg], 1);
        }
      }
      if (!cache) __syncthreads();
    }
    __syncthreads();
    if (pass == 0 && tid == 0) {
      double z = 0.0;
      for (int dg = 255; dg >= 0; --dg) z += (double)hist[dg];
      sh_z = z;
      double target;
      if (topk) {
        int k = tab.k_per_row[(size_t)(tab.item0 + it) * tab.rows_per_item + r];
        k = k < 1 ? 1 : (k > L ? L : k);
        target = (double)k;
      } else {
        target = (double)tab.p * z;
      }
      sh_target = target;
    }
    if (pass == 0) __syncthreads();
    if (wave == 0) {
      double above = sh_above;
      const int pick = pick_digit_wave(hist, cnt, above, sh_target, lane);
      if (lane == 0) {
        sh_prefix = (prefix << 8) | (uint32_t)pick;
        sh_above = above;
        sh_ties = cnt[pick];
      }
    }
    __syncthreads();
  }

  uint32_t tau = 0u;
  int take = 0, ties = 0;
  if (!keep_all) {
    if (tid == 0) {
      const double w_tau = (double)fixed_weight(from_ordered_bits(sh_prefix));
      const double need = sh_target - sh_above;
      int n = w_tau > 0.0 ? (int)fmin(ceil(need / w_tau), 2.0e9) : sh_ties;
      n = n < 1 ? 1 : (n > sh_ties ? sh_ties : n);
      sh_take = n;
      sh_tie_base = 0;
    }
    __syncthreads();
    tau = sh_prefix;
    take = sh_take;
    ties = sh_ties;
  }
  if (tid == 0) {
    const size_t gr = (size_t)(tab.item0 + it) * tab.rows_per_item + r;
    if (tab.row_max) tab.row_max[gr] = m;
    if (tab.row_sum) tab.row_sum[gr] = topk ? (float)sh_z : (float)(sh_z / kSelFix);
  }

  // ---- pass 5: emit the row's bit mask, kSelThreads keys per step, in position order
  uint32_t *mrow = tab.rowmask + I.mask_off + (long long)r * I.W;
  const int n_steps = (I.W * 32 + kSelThreads - 1) / kSelThreads;
  const bool rank_ties = !keep_all && take < ties;
  for (int step = 0; step < n_steps; ++step) {
    const int t = step * kSelThreads + tid;
    if (!keep_all && !cache) {
      fill_tile(step * kSelThreads);
      __syncthreads();
    }
    bool sel = false, tie = false;
    if (t < L) {
      if (keep_all) {
        sel = true;
      } else {
        const uint32_t u = ordered_bits(cache ? cache[t] : lg[tid]);
        sel = u > tau;
        tie = u == tau;
      }
    }
    if (tie && !rank_ties) sel = true;
    if (rank_ties) {
      // position-ordered rank of this tie among all ties of the row
      const unsigned long long bal = __ballot(tie);
      const int before = __popcll(bal & ((1ull << lane) - 1ull));
      if (lane == 0) red_i[wave] = __popcll(bal);
      __syncthreads();
      int base = sh_tie_base, all = 0;
      for (int w = 0; w < NW; ++w) {
        if (w < wave) base += red_i[w];
        all += red_i[w];
      }
      if (tie && base + before < take) sel = true;
      __syncthreads();
      if (tid == 0) sh_tie_base += all;
    }
    const unsigned long long bits = __ballot(sel);
    const int w0 = (step * kSelThreads + wave * 64) >> 5;
    if (lane == 0) {
      if (w0 < I.W) mrow[w0] = (uint32_t)bits;
      if (w0 + 1 < I.W) mrow[w0 + 1] = (uint32_t)(bits >> 32);
    }
    __syncthreads();
  }
}

// grid: every row of the batch (row_list null), or a fixed number of workgroups walking the list
template <typename T>
__global__ __launch_bounds__(kSelThreads) void select_row_kernel(const ScoreTable tab) {
  // workgroup b may keep a row's logits in the b-th slice of the logit cache, if there is one for it
  float *cache = (int)blockIdx.x < tab.cache_rows ? tab.lg_cache + (size_t)blockIdx.x * tab.cache_stride : nullptr;
  if (tab.row_list == nullptr) {
    select_row_body<T>(tab, blockIdx.x, cache);
    return;
  }
  const int n = *tab.n_list;
  for (int i = blockIdx.x; i < n; i += gridDim.x) {
    select_row_body<T>(tab, tab.row_list[i], cache);
    __syncthreads();
  }
}

}  // namespace

// Logit cache of the general selector: room for kCacheRows rows of the longest item (rows beyond that
// recompute their logits in every pass).
constexpr int kCacheRows = 128;
size_t general_cache_bytes(const gvote_item *items, int n_items) {
  int max_L = 0;
  for (int i = 0; i < n_items; ++i) max_L = items[i].L > max_L ? items[i].L : max_L;
  return (size_t)kCacheRows * ((max_L + 63) / 64 * 64) * sizeof(float);
}

ScorePlan plan_score(const gvote_shape *sh, const gvote_item *items, int n_items, int S) {
  ScorePlan p;
  p.ws_bytes = general_cache_bytes(items, n_items) + 256;
  if (fast_path_ok(sh, S, GVOTE_SELECT_TOPP, 0.5f)) p.ws_bytes += plan_fast(sh, items, n_items, S).ws_bytes;
  return p;
}

gvote_status launch_select_rows_general(const gvote_shape *sh, const gvote_item *items, int nb, int item0, int S,
                                        const void *q, float p, int mode, const int *k_per_row, uint32_t *rowmask,
                                        long long mask_off0, float *row_max, float *row_sum, const int *row_list,
                                        const int *n_list, int *n_fallback, float *lg_cache, size_t cache_bytes,
                                        hipStream_t st) {
  ScoreTable tab;
  tab.n_items = nb; tab.S = S; tab.n_q_heads = sh->n_q_heads; tab.n_kv_heads = sh->n_kv_heads;
  tab.head_dim = sh->head_dim; tab.mode = mode; tab.rows_per_item = S * sh->n_q_heads; tab.item0 = item0;
  tab.p = p; tab.pad2 = 0.f; tab.scale = 1.0 / sqrt((double)sh->head_dim);
  tab.q = q; tab.k_per_row = k_per_row; tab.rowmask = rowmask; tab.row_max = row_max; tab.row_sum = row_sum;
  tab.row_list = row_list; tab.n_list = n_list; tab.n_fallback = n_fallback;
  int max_L = 0;
  for (int i = 0; i < nb; ++i) max_L = items[i].L > max_L ? items[i].L : max_L;
  tab.cache_stride = (max_L + 63) / 64 * 64;
  tab.lg_cache = lg_cache;
  tab.cache_rows = lg_cache ? (int)std::min<size_t>(cache_bytes / ((size_t)tab.cache_stride * sizeof(float)), 1 << 20) : 0;
  long long mask_off = mask_off0;
  for (int i = 0; i < nb; ++i) {
    const gvote_item &g = items[i];
    ScoreItem &c = tab.it[i];
    c.k = g.k; c.tok_stride = g.kv_tok_stride; c.head_stride = g.kv_head_stride;
    c.L = g.L; c.W = (g.L + 31) / 32; c.mask_off = mask_off; c.row0 = i * tab.rows_per_item; c.pad = 0;
    mask_off += (long long)tab.rows_per_item * c.W;
  }
  const int all_rows = nb * tab.rows_per_item;
  const dim3 grid(row_list ? (all_rows < 1024 ? all_rows : 1024) : all_rows);
  if (sh->dtype == GVOTE_F32)
    hipLaunchKernelGGL(select_row_kernel<float>, grid, dim3(kSelThreads), 0, st, tab);
  else
    hipLaunchKernelGGL(select_row_kernel<bf16_t>, grid, dim3(kSelThreads), 0, st, tab);
  GVOTE_CHECK_LAUNCH();
  return GVOTE_OK;
}

gvote_status launch_score_select(const gvote_shape *sh, const gvote_item *items, int n_items, int S, const void *q,
                                 float p, int mode, const int *k_per_row, uint32_t *rowmask, float *row_max,
                                 float *row_sum, void *ws, size_t ws_bytes, hipStream_t st) {
  (void)ws_bytes;
  bool fast = fast_path_ok(sh, S, mode, p);
  for (int i = 0; i < n_items && fast; ++i) fast = items[i].L >= 32;   // the matrix-core path loads whole 32-key tiles
  if (fast) return launch_score_fast(sh, items, n_items, S, q, p, mode, k_per_row, rowmask, row_max, row_sum, ws, st);
  long long mask_off = 0;
  const size_t cache_bytes = ws ? general_cache_bytes(items, n_items) : 0;
  for (int b0 = 0; b0 < n_items; b0 += kMaxItems) {
    const int nb = n_items - b0 < kMaxItems ? n_items - b0 : kMaxItems;
    const gvote_status stt = launch_select_rows_general(sh, items + b0, nb, b0, S, q, p, mode, k_per_row, rowmask,
                                                        mask_off, row_max, row_sum, nullptr, nullptr, nullptr,
                                                        reinterpret_cast<float *>(ws), cache_bytes, st);
    if (stt != GVOTE_OK) return stt;
    for (int i = 0; i < nb; ++i) mask_off += (long long)S * sh->n_q_heads * ((items[b0 + i].L + 31) / 32);
  }
  return GVOTE_OK;
}

}  // namespace gvote
