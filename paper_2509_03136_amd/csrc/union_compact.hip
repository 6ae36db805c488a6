// Stage 4 - voting, budget and pruning (paper Sec. 3.2 Step 4; Alg. 1 "K <- union of C^(s)",
// "prune (K, V) to the indices in K"; Sec. 3.4: per-sample masks, one OR, nonzero, gather).
//
//   union_count   OR of the S*G row masks of each KV head, word by word; popcount per chunk of
//                 64 words (2048 tokens).
//   scan_chunks   one workgroup: exclusive prefix sum of the chunk counts in (item, head, chunk)
//                 order -> row offset of every chunk, budget B and offsets per (item, head),
//                 overflow flag.
//   gather        one workgroup per chunk: expand the chunk's bits into an ordered list of kept
//                 positions in LDS, then copy the K and V rows with 16-byte lanes (a 256-byte row
//                 is 16 lanes), rows in ascending position: a stable stream compaction.
// Everything here is integer / byte work and bit-exact by construction.
#include <mutex>

#include "gvote_internal.hpp"

// Scratch memory of the entry point that allocates nothing (gvote_union_compact_static): chunk counts,
// chunk bases and first-chunk indices of one call.  One copy per GPU the library runs on, held until the
// process ends; in host code this name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[gvote::kStaticScratchBytes];

namespace gvote {

namespace {

constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];      // device address of `scratch` on each device, looked up once
std::mutex g_scratch_mutex;

// grid: one workgroup of four waves per chunk; each wave ORs a quarter of the group's rows, wave 0 combines
__global__ __launch_bounds__(256) void union_count_kernel(const UnionTable tab) {
  __shared__ uint32_t part[4][64];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chunk = blockIdx.x;                       // within this batch
  const int it = item_of_chunk(tab, chunk, tab.it[0].chunk0);
  const UnionItem I = tab.it[it];
  const int local = chunk - (I.chunk0 - tab.it[0].chunk0);
  if (it == tab.n_items - 1 && local >= I.n_chunks * tab.n_kv_heads) return;
  const int kvh = local / I.n_chunks, c = local - kvh * I.n_chunks;
  const int G = tab.n_q_heads / tab.n_kv_heads;
  const int word = c * kChunkWords + lane;
  uint32_t acc = 0u;
  if (word < I.W) {
    const uint32_t *rm = tab.rowmask + I.rowmask_off + word;
    // this wave's share of the S*G rows of the group, eight loads in flight at a time
    const int n_rows = tab.S * G;
    const int per_wave = (n_rows + 3) / 4;
    const int i_end = min(n_rows, (wave + 1) * per_wave);
    for (int i0 = wave * per_wave; i0 < i_end; i0 += 8) {
      uint32_t v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        const int i = min(i0 + u, i_end - 1);           // the last row is simply read again
        const int s = i / G, g = i - s * G;
        v[u] = rm[(long long)(s * tab.n_q_heads + kvh * G + g) * I.W];
      }
#pragma unroll
      for (int u = 0; u < 8; ++u) acc |= v[u];
    }
  }
  part[wave][lane] = acc;
  __syncthreads();
  if (wave != 0) return;
  acc = part[0][lane] | part[1][lane] | part[2][lane] | part[3][lane];
  if (word < I.W) {
    if (word == I.W - 1 && (I.L & 31)) acc &= (1u << (I.L & 31)) - 1u;   // never trust bits beyond L
    tab.union_mask[I.union_off + (long long)kvh * I.W + word] = acc;
  }
  int n = __popc(acc);
  for (int off = 32; off > 0; off >>= 1) n += __shfl_xor(n, off, 64);
  if (lane == 0) {
    tab.chunk_count[I.chunk0 + local] = n;
    if (c == 0) tab.head_first[(tab.item0 + it) * tab.n_kv_heads + kvh] = I.chunk0 + local;
  }
}

// single workgroup of 1024 threads over the whole call
__global__ __launch_bounds__(1024) void scan_chunks_kernel(const int *chunk_count, long long *chunk_base,
                                                           const int *head_first, int total_chunks, int n_heads,
                                                           int *budget, long long *offsets, long long capacity,
                                                           int *overflow_flag) {
  __shared__ long long wsum[16];
  __shared__ long long carry;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (tid == 0) carry = 0;
  __syncthreads();
  for (int c0 = 0; c0 < total_chunks; c0 += 1024) {
    const int c = c0 + tid;
    const long long v = c < total_chunks ? (long long)chunk_count[c] : 0;
    long long x = v;
    for (int off = 1; off < 64; off <<= 1) {
      const long long y = __shfl_up(x, off, 64);
      if (lane >= off) x += y;
    }
    if (lane == 63) wsum[wave] = x;
    __syncthreads();
    long long base = carry;
    for (int w = 0; w < wave; ++w) base += wsum[w];
    if (c < total_chunks) chunk_base[c] = base + x - v;
    __syncthreads();
    if (tid == 1023) carry = base + x;
    __syncthreads();
  }
  if (tid == 0) {
    chunk_base[total_chunks] = carry;
    offsets[n_heads] = carry;
    *overflow_flag = carry > capacity ? 1 : 0;
  }
  __syncthreads();
  const long long total = carry;
  for (int hh = tid; hh < n_heads; hh += 1024) {
    const long long b0 = chunk_base[head_first[hh]];
    const long long b1 = hh + 1 < n_heads ? chunk_base[head_first[hh + 1]] : total;
    offsets[hh] = b0;
    budget[hh] = (int)(b1 - b0);
  }
}

// grid: one workgroup per chunk of this batch
template <typename T>
__global__ __launch_bounds__(256) void gather_kernel(const UnionTable tab) {
  const int chunk = blockIdx.x;
  const int it = item_of_chunk(tab, chunk, tab.it[0].chunk0);
  const UnionItem I = tab.it[it];
  const int local = chunk - (I.chunk0 - tab.it[0].chunk0);
  const int kvh = local / I.n_chunks, c = local - kvh * I.n_chunks;
  const int tid = threadIdx.x;

  __shared__ int list[kChunkWords * 32];
  __shared__ int n_kept;
  if (tid < 64) {   // wave 0: per-word exclusive prefix of popcounts, then expand bits in order
    const int word = c * kChunkWords + tid;
    const uint32_t bits = word < I.W ? tab.union_mask[I.union_off + (long long)kvh * I.W + word] : 0u;
    const int n = __popc(bits);
    int x = n;
    for (int off = 1; off < 64; off <<= 1) {
      const int y = __shfl_up(x, off, 64);
      if (tid >= off) x += y;
    }
    int pos = x - n;
    uint32_t b = bits;
    while (b) {
      const int bit = __ffs(b) - 1;
      list[pos++] = word * 32 + bit;
      b &= b - 1;
    }
    if (tid == 63) n_kept = x;
  }
  __syncthreads();
  const int n = n_kept;
  const long long base = tab.chunk_base[I.chunk0 + local];
  const int dk = tab.head_dim;
  const int ppr = dk * (int)sizeof(T) / 16;      // 16-byte pieces per row
  const int rows_per_step = 256 / ppr;
  const int piece = tid % ppr, rsel = tid / ppr;
  const T *kb = reinterpret_cast<const T *>(I.k) + (long long)kvh * I.head_stride;
  const T *vb = reinterpret_cast<const T *>(I.v) + (long long)kvh * I.head_stride;
  T *ko = reinterpret_cast<T *>(tab.k_out);
  T *vo = reinterpret_cast<T *>(tab.v_out);
  constexpr int EPP = 16 / (int)sizeof(T);       // elements per piece
  if (rsel < rows_per_step) {
    // kept rows are read once and written once: non-temporal both ways, the caches stay with W_q.  Four rows per
    // thread are in flight before the first is written.
    constexpr int U = 4;
    for (int i0 = rsel; i0 < n; i0 += U * rows_per_step) {
      int t[U];
      u32x4_t kx[U], vx[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = i0 + u * rows_per_step;
        t[u] = list[i < n ? i : n - 1];
        const long long src = (long long)t[u] * I.tok_stride + piece * EPP;
        kx[u] = load_stream16(kb + src);
        vx[u] = load_stream16(vb + src);
      }
#pragma unroll
      for (int u = 0; u < U; ++u) {
        const int i = i0 + u * rows_per_step;
        const long long dst = base + i;
        if (i < n && dst < tab.capacity) {
          __builtin_nontemporal_store(kx[u], reinterpret_cast<u32x4_t *>(ko + dst * dk + piece * EPP));
          __builtin_nontemporal_store(vx[u], reinterpret_cast<u32x4_t *>(vo + dst * dk + piece * EPP));
          if (piece == 0 && tab.idx_out) tab.idx_out[dst] = t[u];
        }
      }
    }
  }
}

// one wave per row: popcount of the row's words; grid (ceil(rows / 4)), item geometry by value
struct CountTable {
  int n_items, rows_per_item, repeat, item0;
  const uint32_t *rowmask;
  int *counts;
  long long mask_off[kMaxItems];
  int W[kMaxItems];
};
__global__ __launch_bounds__(256) void count_rows_kernel(const CountTable tab) {
  const int lane = threadIdx.x & 63;
  const int grow = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (grow >= tab.n_items * tab.rows_per_item) return;
  const int it = grow / tab.rows_per_item, r = grow - it * tab.rows_per_item;
  const uint32_t *row = tab.rowmask + tab.mask_off[it] + (long long)r * tab.W[it];
  int n = 0;
  for (int w = lane; w < tab.W[it]; w += 64) n += __popc(row[w]);
  for (int off = 32; off > 0; off >>= 1) n += __shfl_xor(n, off, 64);
  if (lane == 0)
    for (int c = 0; c < tab.repeat; ++c)
      tab.counts[((size_t)(tab.item0 + it) * tab.repeat + c) * tab.rows_per_item + r] = n;
}

}  // namespace

gvote_status launch_count_rows(const gvote_shape *sh, const gvote_item *items, int n_items, int S,
                               const uint32_t *rowmask, int repeat, int *counts, hipStream_t st) {
  long long off = 0;
  for (int b0 = 0; b0 < n_items; b0 += kMaxItems) {
    const int nb = n_items - b0 < kMaxItems ? n_items - b0 : kMaxItems;
    CountTable tab;
    tab.n_items = nb; tab.rows_per_item = S * sh->n_q_heads; tab.repeat = repeat; tab.item0 = b0;
    tab.rowmask = rowmask; tab.counts = counts;
    for (int i = 0; i < nb; ++i) {
      tab.W[i] = (items[b0 + i].L + 31) / 32;
      tab.mask_off[i] = off;
      off += (long long)tab.rows_per_item * tab.W[i];
    }
    hipLaunchKernelGGL(count_rows_kernel, dim3(ceil_div(nb * tab.rows_per_item, 4)), dim3(256), 0, st, tab);
    GVOTE_CHECK_LAUNCH();
  }
  return GVOTE_OK;
}

gvote_status static_scratch_of_current_device(void **ptr) {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess) return GVOTE_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return GVOTE_ERR_CAPACITY;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return GVOTE_ERR_HIP;
    g_scratch_ptr[dev] = p;
  }
  *ptr = g_scratch_ptr[dev];
  return GVOTE_OK;
}

UnionPlan plan_union(const gvote_shape *sh, const gvote_item *items, int n_items) {
  UnionPlan p;
  long long chunks = 0;
  for (int i = 0; i < n_items; ++i)
    chunks += (long long)sh->n_kv_heads * ceil_div((items[i].L + 31) / 32, kChunkWords);
  p.total_chunks = (int)chunks;
  p.off_base = align_up((size_t)chunks * sizeof(int), 256);
  p.off_head = p.off_base + align_up(((size_t)chunks + 1) * sizeof(long long), 256);
  p.ws_bytes = p.off_head + align_up(((size_t)n_items * sh->n_kv_heads + 1) * sizeof(int), 256);
  return p;
}

gvote_status launch_union_compact(const gvote_shape *sh, const gvote_item *items, int n_items, int S,
                                  const uint32_t *rowmask, uint32_t *union_mask, int *budget, long long *offsets,
                                  void *k_out, void *v_out, int *idx_out, long long capacity, int *overflow_flag,
                                  void *ws, hipStream_t st) {
  const UnionPlan plan = plan_union(sh, items, n_items);
  char *wsb = reinterpret_cast<char *>(ws);
  UnionTable tab;
  tab.S = S; tab.n_q_heads = sh->n_q_heads; tab.n_kv_heads = sh->n_kv_heads; tab.head_dim = sh->head_dim;
  tab.total_chunks_call = plan.total_chunks; tab.n_heads_call = n_items * sh->n_kv_heads;
  tab.rowmask = rowmask; tab.union_mask = union_mask;
  tab.chunk_count = reinterpret_cast<int *>(wsb);
  tab.chunk_base = reinterpret_cast<long long *>(wsb + plan.off_base);
  tab.head_first = reinterpret_cast<int *>(wsb + plan.off_head);
  tab.k_out = k_out; tab.v_out = v_out; tab.idx_out = idx_out; tab.capacity = capacity;

  const int rows_per_item = S * sh->n_q_heads;
  // pass 1 over the batches: union + counts; pass 2: one scan; pass 3 over the batches: gather
  for (int phase = 0; phase < 2; ++phase) {
    long long rm_off = 0, un_off = 0;
    int chunk0 = 0;
    for (int b0 = 0; b0 < n_items; b0 += kMaxItems) {
      const int nb = n_items - b0 < kMaxItems ? n_items - b0 : kMaxItems;
      tab.n_items = nb;
      tab.item0 = b0;
      int batch_chunks = 0;
      for (int i = 0; i < nb; ++i) {
        const gvote_item &g = items[b0 + i];
        UnionItem &u = tab.it[i];
        u.k = g.k; u.v = g.v; u.tok_stride = g.kv_tok_stride; u.head_stride = g.kv_head_stride;
        u.L = g.L; u.W = (g.L + 31) / 32;
        u.rowmask_off = rm_off; u.union_off = un_off;
        u.n_chunks = ceil_div(u.W, kChunkWords);
        u.chunk0 = chunk0 + batch_chunks;
        rm_off += (long long)rows_per_item * u.W;
        un_off += (long long)sh->n_kv_heads * u.W;
        batch_chunks += u.n_chunks * sh->n_kv_heads;
      }
      if (phase == 0) {
        hipLaunchKernelGGL(union_count_kernel, dim3(batch_chunks), dim3(256), 0, st, tab);
      } else if (sh->dtype == GVOTE_F32) {
        hipLaunchKernelGGL(gather_kernel<float>, dim3(batch_chunks), dim3(256), 0, st, tab);
      } else {
        hipLaunchKernelGGL(gather_kernel<bf16_t>, dim3(batch_chunks), dim3(256), 0, st, tab);
      }
      GVOTE_CHECK_LAUNCH();
      chunk0 += batch_chunks;
    }
    if (phase == 0) {
      hipLaunchKernelGGL(scan_chunks_kernel, dim3(1), dim3(1024), 0, st, tab.chunk_count, tab.chunk_base,
                         tab.head_first, plan.total_chunks, n_items * sh->n_kv_heads, budget, offsets, capacity,
                         overflow_flag);
      GVOTE_CHECK_LAUNCH();
    }
  }
  return GVOTE_OK;
}

}  // namespace gvote
