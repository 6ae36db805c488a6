// Stage 1 - Gaussian fit of the prefill hidden states (paper Sec. 3.2 Step 2; Alg. 1, the
// "mean(h), var(h)" line): per-channel mean and variance over tokens n_s .. L-1.
//
// One pass over hidden[L, d], the largest stream of the whole path (d * elem bytes per token),
// so the kernel is a pure HBM reader: every wave loads 1 KiB contiguous pieces of a row
// (64 lanes x 16 B), four waves of a workgroup take interleaved rows, eight rows are in flight
// per lane.  Sums are taken about a pivot row (shifted data) in fp32 per row chunk, chunks are
// merged in fp64 in a fixed order (Chan et al. pairwise update) -> deterministic output.
#include "gvote_internal.hpp"

namespace gvote {

namespace {

constexpr int kFitThreads = 256;
constexpr int kFitUnroll = 8;

template <typename T>
__global__ __launch_bounds__(kFitThreads) void moments_partial_kernel(const FitTable tab) {
  constexpr int NV = Vec16<T>::N;
  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int chunk = blockIdx.y;
  const int it = item_of_chunk(tab, chunk, 0);
  const FitItem I = tab.it[it];
  const int col = (blockIdx.x * 64 + lane) * NV;
  const bool active = col < tab.d;
  const int r0 = I.n_skip + (chunk - I.chunk0) * tab.rows_per_chunk;
  const int r1 = min(I.L, r0 + tab.rows_per_chunk);
  const T *base = reinterpret_cast<const T *>(I.hidden) + col;

  float pivot[NV], s[NV], ss[NV];
#pragma unroll
  for (int i = 0; i < NV; ++i) { pivot[i] = 0.f; s[i] = 0.f; ss[i] = 0.f; }
  if (active) {
    Vec16<T>::load(base + (long long)r0 * I.stride, pivot);
    // main loop without any guard (straight-line loads keep all eight rows in flight), then a remainder
    int r = r0 + wave;
    for (; r + 4 * (kFitUnroll - 1) < r1; r += 4 * kFitUnroll) {
      float x[kFitUnroll][NV];
#pragma unroll
      for (int u = 0; u < kFitUnroll; ++u) Vec16Stream<T>::load(base + (long long)(r + 4 * u) * I.stride, x[u]);
#pragma unroll
      for (int u = 0; u < kFitUnroll; ++u) {
#pragma unroll
        for (int i = 0; i < NV; ++i) {
          const float dlt = x[u][i] - pivot[i];
          s[i] += dlt;
          ss[i] = fmaf(dlt, dlt, ss[i]);
        }
      }
    }
    for (; r < r1; r += 4) {
      float x[NV];
      Vec16Stream<T>::load(base + (long long)r * I.stride, x);
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const float dlt = x[i] - pivot[i];
        s[i] += dlt;
        ss[i] = fmaf(dlt, dlt, ss[i]);
      }
    }
  }
  __shared__ float red[3][64][2 * NV];
  if (wave > 0) {
#pragma unroll
    for (int i = 0; i < NV; ++i) { red[wave - 1][lane][i] = s[i]; red[wave - 1][lane][NV + i] = ss[i]; }
  }
  __syncthreads();
  if (wave == 0 && active) {
    const float n = (float)(r1 - r0);
    float *pm = tab.partial + ((size_t)chunk * 2) * tab.d + col;
    float *pv = pm + tab.d;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const float st = s[i] + red[0][lane][i] + red[1][lane][i] + red[2][lane][i];
      const float sst = ss[i] + red[0][lane][NV + i] + red[1][lane][NV + i] + red[2][lane][NV + i];
      pm[i] = pivot[i] + st / n;
      pv[i] = fmaxf(0.f, sst - st * st / n);
    }
  }
}

// Chan merge of the chunks in fp64, in a fixed order: 32 channels per workgroup, eight threads per channel each merge
// every eighth chunk, then thread 0 of the channel merges the eight partial results (a long single item has hundreds of
// chunks: one thread walking them all took longer than the pass over the hidden states).
constexpr int kFinCh = 32, kFinLanes = 8;
__device__ __forceinline__ void chan_merge(double &n, double &mean, double &m2, double nb, double mb, double vb) {
  if (nb <= 0.0) return;
  const double nn = n + nb, delta = mb - mean, r = nb / nn;
  mean += delta * r;
  m2 += vb + delta * delta * (n * r);
  n = nn;
}
__global__ __launch_bounds__(kFinCh * kFinLanes) void moments_finalize_kernel(const FitTable tab, int ddof, float *mu,
                                                                             float *var, int item0) {
  __shared__ double sn[kFinLanes][kFinCh], smean[kFinLanes][kFinCh], sm2[kFinLanes][kFinCh];
  const int it = blockIdx.y;
  const int ch = threadIdx.x % kFinCh, cl = threadIdx.x / kFinCh;
  const int col = blockIdx.x * kFinCh + ch;
  const FitItem I = tab.it[it];
  double n = 0.0, mean = 0.0, m2 = 0.0;
  if (col < tab.d) {
    for (int c = cl; c < I.n_chunks; c += kFinLanes) {
      const int r0 = I.n_skip + c * tab.rows_per_chunk;
      const double nb = (double)(min(I.L, r0 + tab.rows_per_chunk) - r0);
      const float *pm = tab.partial + ((size_t)(I.chunk0 + c) * 2) * tab.d + col;
      chan_merge(n, mean, m2, nb, (double)pm[0], (double)pm[tab.d]);
    }
  }
  sn[cl][ch] = n; smean[cl][ch] = mean; sm2[cl][ch] = m2;
  __syncthreads();
  if (cl != 0 || col >= tab.d) return;
  for (int l = 1; l < kFinLanes; ++l) chan_merge(n, mean, m2, sn[l][ch], smean[l][ch], sm2[l][ch]);
  mu[(size_t)(item0 + it) * tab.d + col] = (float)mean;
  var[(size_t)(item0 + it) * tab.d + col] = (float)(m2 / (n - (double)ddof));
}

}  // namespace

FitPlan plan_fit(const gvote_shape *sh, const gvote_item *items, int n_items) {
  // aim at ~4096 workgroups so that every CU holds several; a chunk is at least 64 rows
  int64_t rows = 0;
  for (int i = 0; i < n_items; ++i) rows += items[i].L - items[i].n_skip;
  const int nv = sh->dtype == GVOTE_F32 ? 4 : 8;
  const int colblocks = ceil_div(sh->d_model, 64 * nv);
  int64_t rpc = (rows * colblocks + 2047) / 2048;
  rpc = (rpc + 31) / 32 * 32;
  if (rpc < 64) rpc = 64;
  if (rpc > 4096) rpc = 4096;
  FitPlan p;
  p.rows_per_chunk = (int)rpc;
  p.total_chunks = 0;
  p.max_batch_chunks = 0;
  long long in_batch = 0;
  for (int i = 0; i < n_items; ++i) {
    if (i % kMaxItems == 0) in_batch = 0;
    const int c = ceil_div(items[i].L - items[i].n_skip, rpc);
    p.total_chunks += c;
    in_batch += c;
    if (in_batch > p.max_batch_chunks) p.max_batch_chunks = in_batch;
  }
  p.ws_bytes = (size_t)p.total_chunks * 2 * sh->d_model * sizeof(float);
  return p;
}

gvote_status launch_fit(const gvote_shape *sh, const gvote_item *items, int n_items, int ddof, float *mu, float *var,
                        void *ws, hipStream_t st) {
  const FitPlan plan = plan_fit(sh, items, n_items);
  const int nv = sh->dtype == GVOTE_F32 ? 4 : 8;
  const int colblocks = ceil_div(sh->d_model, 64 * nv);
  int chunk_done = 0;
  for (int b0 = 0; b0 < n_items; b0 += kMaxItems) {
    const int nb = n_items - b0 < kMaxItems ? n_items - b0 : kMaxItems;
    FitTable tab;
    tab.n_items = nb;
    tab.d = sh->d_model;
    tab.rows_per_chunk = plan.rows_per_chunk;
    tab.pad = 0;
    tab.partial = reinterpret_cast<float *>(ws) + (size_t)chunk_done * 2 * sh->d_model;
    int c = 0;
    for (int i = 0; i < nb; ++i) {
      const gvote_item &g = items[b0 + i];
      FitItem &f = tab.it[i];
      f.hidden = g.hidden;
      f.stride = g.hidden_row_stride;
      f.L = g.L;
      f.n_skip = g.n_skip;
      f.chunk0 = c;
      f.n_chunks = ceil_div(g.L - g.n_skip, plan.rows_per_chunk);
      c += f.n_chunks;
    }
    if (c > kMaxFitChunks) return GVOTE_ERR_CAPACITY;   // (the entry point has already checked the plan)
    const dim3 grid(colblocks, c);
    if (sh->dtype == GVOTE_F32)
      hipLaunchKernelGGL(moments_partial_kernel<float>, grid, dim3(kFitThreads), 0, st, tab);
    else
      hipLaunchKernelGGL(moments_partial_kernel<bf16_t>, grid, dim3(kFitThreads), 0, st, tab);
    GVOTE_CHECK_LAUNCH();
    hipLaunchKernelGGL(moments_finalize_kernel, dim3(ceil_div(sh->d_model, kFinCh), nb), dim3(kFinCh * kFinLanes), 0, st, tab,
                       ddof, mu, var, b0);
    GVOTE_CHECK_LAUNCH();
    chunk_done += c;
  }
  return GVOTE_OK;
}

}  // namespace gvote
