// Stage 3, bf16 fast path - K-streaming scores on the matrix cores and a histogram search for the
// mass-p cut (paper Eq. (1) logits and softmax weights; Sec. 3.1 minimal key set of mass p).
//
// Nothing of size S*H_q*L is stored: logits are recomputed from K in each pass, bit-identically
// (same MFMA sequence), and only per-row statistics travel between the passes.
//
//   score_max    pass A: per (item, KV head, key chunk) the maximum raw dot product of every
//                query row of the group.
//   score_hist   pass B: weight exp(l - m) of every key accumulated into 256 bins of width 1/16
//                in logit units below the row maximum, per row, in LDS; the last bin collects
//                everything further down.
//   find_bin     per row: merge the chunks, Z, target p*Z, walk the bins from the top: the bin
//                a* where the cumulative weight crosses the target, and the weight above it.
//   score_emit   pass C: keys in bins above a* are selected outright (bit masks, transposed in
//                LDS so every row writes whole 128-byte lines); keys inside bin a* are appended
//                (raw dot, position) to the row's candidate list.
//   resolve      per row: exact selection among the candidates - radix search over the 64-bit
//                key (ordered dot, ~position), so ties go to the lower position - and OR of the
//                chosen bits into the mask.
// Rows whose cut falls into the collecting bin, or whose candidate lists overflow, are flagged
// and redone by the exact general selector (select_row_kernel).
//
// A workgroup is 8 waves; a wave owns 32-key tiles.  K rows of a tile are fetched with fully
// coalesced 16-byte lanes (16 lanes per 256-byte row), written to a wave-private, XOR-swizzled
// LDS tile and read back in MFMA operand order; the next tile's global loads are issued before
// the current tile's MFMAs.  v_mfma_f32_32x32x16_bf16: A = 32 keys x 16 channels, B = 16 channels
// x 32 query rows (kept in registers for the whole kernel), C[key][query row]: a lane owns ONE
// query row and 16 keys, so row statistics need no cross-lane traffic inside the loop.
#include "gvote_internal.hpp"

namespace gvote {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

constexpr int kWaves = 8;
constexpr int kThreads = kWaves * 64;
constexpr int kRoundTiles = 4;                         // tiles per wave per emit round
constexpr int kRoundKeys = kWaves * kRoundTiles * 32;  // 1024
constexpr int kLocalCand = 32;                         // LDS candidate slots per row per round

__device__ __forceinline__ uint32_t ordered_bits(float f) {
  const uint32_t b = __float_as_uint(f);
  return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float from_ordered_bits(uint32_t u) {
  return __uint_as_float((u & 0x80000000u) ? (u ^ 0x80000000u) : ~u);
}

// position of accumulator register r of lane (hf = lane / 32) inside the 32-key tile
__device__ __forceinline__ int key_of(int r, int hf) { return 8 * (r >> 2) + 4 * hf + (r & 3); }

struct WgCoord {
  int it, kvh, chunk, qb, n0, t_begin, t_end, slot;
};

__device__ __forceinline__ WgCoord decode_wg(const FastTable &tab, int wg) {
  WgCoord c;
  c.it = 0;
  while (c.it + 1 < tab.n_items && wg >= tab.it[c.it + 1].wg0) ++c.it;
  const FastItem &I = tab.it[c.it];
  int local = wg - I.wg0;
  c.qb = local % tab.NQB;
  local /= tab.NQB;
  c.chunk = local % I.n_chunks;
  c.kvh = local / I.n_chunks;
  c.n0 = c.qb * 64;
  c.t_begin = c.chunk * tab.chunk_keys;
  c.t_end = min(I.L, c.t_begin + tab.chunk_keys);
  c.slot = I.part0 + c.kvh * I.n_chunks + c.chunk;
  return c;
}

template <int DK>
struct Tile {
  static constexpr int KS = DK / 16;            // MFMA k-steps
  static constexpr int PPR = DK / 8;            // 16-byte pieces per key row
  static constexpr int RPL = 64 / PPR;          // key rows covered by one wave-wide load
  static constexpr int LOADS = 32 / RPL;        // wave-wide loads per tile
  static constexpr int BYTES = 32 * DK * 2;

  bf16x8 bq[2][KS];

  __device__ __forceinline__ void load_q(const FastTable &tab, int item, int kvh, int n0, int lane) {
    const int col = lane & 31, hf = lane >> 5;
    const bf16_t *q = reinterpret_cast<const bf16_t *>(tab.q) + (size_t)(tab.item0 + item) * tab.rows_per_item * DK;
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const int n = n0 + 32 * nb + col;
      const bool ok = n < tab.NQ;
      const int s = ok ? n / tab.G : 0, g = ok ? n % tab.G : 0;
      const bf16_t *row = q + (size_t)(s * tab.Hq + kvh * tab.G + g) * DK + 8 * hf;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        uint4 raw = make_uint4(0, 0, 0, 0);
        if (ok) raw = *reinterpret_cast<const uint4 *>(row + 16 * ks);
        bq[nb][ks] = __builtin_bit_cast(bf16x8, raw);
      }
    }
  }

  // coalesced fetch of keys t0 .. t0+31 of one KV head (zeros beyond L)
  __device__ __forceinline__ void fetch(uint4 (&pre)[LOADS], const bf16_t *khead, long long tok_stride, int t0, int L,
                                        int lane) const {
    const int piece = lane % PPR, sub = lane / PPR;
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
      const int t = t0 + j * RPL + sub;
      pre[j] = make_uint4(0, 0, 0, 0);
      if (t < L) pre[j] = *reinterpret_cast<const uint4 *>(khead + (long long)t * tok_stride + piece * 8);
    }
  }

  __device__ __forceinline__ void stage(const uint4 (&pre)[LOADS], unsigned char *lds, int lane) const {
    const int piece = lane % PPR, sub = lane / PPR;
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
      const int key = j * RPL + sub;
      const int phys = piece ^ (key & (PPR - 1));
      *reinterpret_cast<uint4 *>(lds + (key * PPR + phys) * 16) = pre[j];
    }
  }

  __device__ __forceinline__ void compute(floatx16 (&acc)[2], const unsigned char *lds, int lane, bool two) const {
    const int key = lane & 31, hf = lane >> 5;
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc[0][r] = 0.f; acc[1][r] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int phys = (2 * ks + hf) ^ (key & (PPR - 1));
      const uint4 raw = *reinterpret_cast<const uint4 *>(lds + (key * PPR + phys) * 16);
      const bf16x8 a = __builtin_bit_cast(bf16x8, raw);
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[0][ks], acc[0], 0, 0, 0);
      if (two) acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bq[1][ks], acc[1], 0, 0, 0);
    }
  }
};

// ------------------------------------------------------------------ pass A: chunk maxima
template <int DK>
__global__ __launch_bounds__(kThreads) void score_max_kernel(const FastTable tab) {
  __shared__ __align__(16) unsigned char tiles[kWaves][Tile<DK>::BYTES];
  __shared__ uint32_t smax[64];
  const WgCoord c = decode_wg(tab, blockIdx.x);
  const FastItem I = tab.it[c.it];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5;
  if (tid < 64) smax[tid] = 0u;
  Tile<DK> T;
  T.load_q(tab, c.it, c.kvh, c.n0, lane);
  const bool two = c.n0 + 32 < tab.NQ;
  const bf16_t *khead = reinterpret_cast<const bf16_t *>(I.k) + (long long)c.kvh * I.head_stride;
  const int n_tiles = (c.t_end - c.t_begin + 31) >> 5;
  float mx[2] = {-INFINITY, -INFINITY};
  uint4 pre[Tile<DK>::LOADS];
  if (wave < n_tiles) T.fetch(pre, khead, I.tok_stride, c.t_begin + wave * 32, c.t_end, lane);
  __syncthreads();
  for (int tile = wave; tile < n_tiles; tile += kWaves) {
    const int t0 = c.t_begin + tile * 32;
    T.stage(pre, tiles[wave], lane);
    if (tile + kWaves < n_tiles) T.fetch(pre, khead, I.tok_stride, t0 + kWaves * 32, c.t_end, lane);
    __builtin_amdgcn_wave_barrier();
    floatx16 acc[2];
    T.compute(acc, tiles[wave], lane, two);
    __builtin_amdgcn_wave_barrier();
    if (t0 + 32 <= c.t_end) {
#pragma unroll
      for (int r = 0; r < 16; ++r) { mx[0] = fmaxf(mx[0], acc[0][r]); mx[1] = fmaxf(mx[1], acc[1][r]); }
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        if (t0 + key_of(r, hf) < c.t_end) { mx[0] = fmaxf(mx[0], acc[0][r]); mx[1] = fmaxf(mx[1], acc[1][r]); }
      }
    }
  }
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    float v = fmaxf(mx[nb], __shfl_xor(mx[nb], 32, 64));
    if (lane < 32) atomicMax(&smax[32 * nb + lane], ordered_bits(v));
  }
  __syncthreads();
  if (tid < 64 && c.n0 + tid < tab.NQ)
    tab.part_max[(size_t)c.slot * tab.NQ + c.n0 + tid] = from_ordered_bits(smax[tid]);
}

// ------------------------------------------------------------------ pass B: weight histograms
template <int DK>
__global__ __launch_bounds__(kThreads) void score_hist_kernel(const FastTable tab) {
  __shared__ __align__(16) unsigned char tiles[kWaves][Tile<DK>::BYTES];
  __shared__ float hist[64 * (kBins + 1)];
  __shared__ float s_ref[64];
  __shared__ int s_top[64];
  const WgCoord c = decode_wg(tab, blockIdx.x);
  const FastItem I = tab.it[c.it];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, col = lane & 31;
  for (int i = tid; i < 64 * (kBins + 1); i += kThreads) hist[i] = 0.f;
  if (tid < 64) {
    float m = -INFINITY;
    if (c.n0 + tid < tab.NQ) {
      const float *pm = tab.part_max + (size_t)(I.part0 + c.kvh * I.n_chunks) * tab.NQ + c.n0 + tid;
      for (int ch = 0; ch < I.n_chunks; ++ch) m = fmaxf(m, pm[(size_t)ch * tab.NQ]);
    }
    s_ref[tid] = m * tab.c2;
    s_top[tid] = (int)floorf(m * tab.c1);
  }
  Tile<DK> T;
  T.load_q(tab, c.it, c.kvh, c.n0, lane);
  const bool two = c.n0 + 32 < tab.NQ;
  const bf16_t *khead = reinterpret_cast<const bf16_t *>(I.k) + (long long)c.kvh * I.head_stride;
  const int n_tiles = (c.t_end - c.t_begin + 31) >> 5;
  uint4 pre[Tile<DK>::LOADS];
  if (wave < n_tiles) T.fetch(pre, khead, I.tok_stride, c.t_begin + wave * 32, c.t_end, lane);
  __syncthreads();
  const int nblk = two ? 2 : 1;
  float ref[2];
  int top[2];
  float *hrow[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    ref[nb] = s_ref[32 * nb + col];
    top[nb] = s_top[32 * nb + col];
    hrow[nb] = hist + (32 * nb + col) * (kBins + 1);
  }
  const float c1 = tab.c1, c2 = tab.c2;
  // raw dot below which a key falls into the collecting (last) bin: those are summed in a register
  float dtail[2], tail[2] = {0.f, 0.f};
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const bool ok = c.n0 + 32 * nb + col < tab.NQ;
    dtail[nb] = ok ? ((float)(top[nb] - (kBins - 2)) - 0.5f) / c1 : INFINITY;
    if (!ok) ref[nb] = INFINITY;     // weight exp2(-inf) = 0 for rows that do not exist
  }
  auto hist_add = [&](float d, int nb) {
    const float w = __builtin_amdgcn_exp2f(fmaf(d, c2, -ref[nb]));
    // floor(d * c1) is the authority on the bin; the register shortcut is only taken when the key is
    // surely at or beyond the last bin (d < dtail - margin), anything near the edge goes the exact way
    if (d < dtail[nb]) {
      tail[nb] += w;
    } else {
      const int a = (int)floorf(d * c1);
      const int j = min(top[nb] - a, kBins - 1);
      atomicAdd(hrow[nb] + j, w);
    }
  };
  for (int tile = wave; tile < n_tiles; tile += kWaves) {
    const int t0 = c.t_begin + tile * 32;
    T.stage(pre, tiles[wave], lane);
    if (tile + kWaves < n_tiles) T.fetch(pre, khead, I.tok_stride, t0 + kWaves * 32, c.t_end, lane);
    __builtin_amdgcn_wave_barrier();
    floatx16 acc[2];
    T.compute(acc, tiles[wave], lane, two);
    __builtin_amdgcn_wave_barrier();
    if (t0 + 32 <= c.t_end) {
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        if (nb < nblk) {
#pragma unroll
          for (int r = 0; r < 16; ++r) hist_add(acc[nb][r], nb);
        }
      }
    } else {
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        if (nb < nblk) {
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (t0 + key_of(r, hf) < c.t_end) hist_add(acc[nb][r], nb);
        }
      }
    }
  }
  // the collecting bin was kept in registers; lanes of rows that do not exist hold zeros
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    const float v = tail[nb] + __shfl_xor(tail[nb], 32, 64);
    if (lane < 32 && c.n0 + 32 * nb + col < tab.NQ) atomicAdd(hrow[nb] + (kBins - 1), v);
  }
  __syncthreads();
  float *out = tab.part_hist + ((size_t)c.slot * tab.NQ + c.n0) * kBins;
  const int rows = min(64, tab.NQ - c.n0);
  for (int i = tid; i < rows * kBins; i += kThreads) out[i] = hist[(i / kBins) * (kBins + 1) + (i % kBins)];
}

// ------------------------------------------------------------------ per row: bin of the cut.  grid = rows, 256 threads
__global__ __launch_bounds__(kBins) void find_bin_kernel(const FastTable tab) {
  const int grow = blockIdx.x;
  const int it = grow / tab.rows_per_item, r = grow - it * tab.rows_per_item;
  const int s = r / tab.Hq, h = r - s * tab.Hq;
  const int kvh = h / tab.G, g = h - kvh * tab.G;
  const int n = s * tab.G + g;
  const FastItem I = tab.it[it];
  const int j = threadIdx.x, lane = j & 63, wave = j >> 6;
  const size_t slot0 = (size_t)(I.part0 + kvh * I.n_chunks);
  double mine = 0.0;
  float m = -INFINITY;
  for (int ch = 0; ch < I.n_chunks; ++ch) {
    mine += (double)tab.part_hist[((slot0 + ch) * tab.NQ + n) * kBins + j];
    m = fmaxf(m, tab.part_max[(slot0 + ch) * tab.NQ + n]);
  }
  // inclusive scan over bins (bin 0 = highest logits)
  __shared__ double wsum[4];
  double x = mine;
  for (int off = 1; off < 64; off <<= 1) {
    const double y = __shfl_up(x, off, 64);
    if (lane >= off) x += y;
  }
  if (lane == 63) wsum[wave] = x;
  __syncthreads();
  double base = 0.0;
  for (int w = 0; w < wave; ++w) base += wsum[w];
  const double cum = base + x;
  const double Z = wsum[0] + wsum[1] + wsum[2] + wsum[3];
  const double target = (double)tab.p * Z;
  const double before = cum - mine;
  RowInfo *info = tab.info + grow;
  if (before < target && cum >= target) {
    info->mdot = m;
    info->astar = (int)floorf(m * tab.c1) - j;
    info->flag = (j == kBins - 1) ? 1 : 0;
    info->above = before;
    info->target = target;
  }
  if (j == 0) {
    if (grow == 0 && tab.item0 == 0) *tab.n_fallback = 0;
    tab.cand_cnt[grow] = 0;
    const size_t gr = (size_t)(tab.item0 + it) * tab.rows_per_item + r;
    if (tab.row_max) tab.row_max[gr] = m * tab.scale;
    if (tab.row_sum) tab.row_sum[gr] = (float)Z;
  }
}

// ------------------------------------------------------------------ pass C: masks + boundary candidates
template <int DK>
__global__ __launch_bounds__(kThreads) void score_emit_kernel(const FastTable tab) {
  __shared__ __align__(16) unsigned char tiles[kWaves][Tile<DK>::BYTES];
  __shared__ uint32_t mwords[64][kWaves * kRoundTiles + 1];
  __shared__ uint2 cbuf[64][kLocalCand];
  __shared__ int ccnt[64];
  __shared__ int cbase[64];
  __shared__ int s_astar[64];
  const WgCoord c = decode_wg(tab, blockIdx.x);
  const FastItem I = tab.it[c.it];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, hf = lane >> 5, col = lane & 31;
  const int row_base = c.it * tab.rows_per_item;   // batch-local row index of (s = 0, h = 0)
  if (tid < 64) {
    const int n = c.n0 + tid;
    int a = 0x7FFFFFFF;
    if (n < tab.NQ) {
      const int s = n / tab.G, g = n % tab.G;
      a = tab.info[row_base + s * tab.Hq + c.kvh * tab.G + g].astar;
    }
    s_astar[tid] = a;
    ccnt[tid] = 0;
  }
  Tile<DK> T;
  T.load_q(tab, c.it, c.kvh, c.n0, lane);
  const bool two = c.n0 + 32 < tab.NQ;
  const bf16_t *khead = reinterpret_cast<const bf16_t *>(I.k) + (long long)c.kvh * I.head_stride;
  __syncthreads();
  int astar[2];
  astar[0] = s_astar[col];
  astar[1] = s_astar[32 + col];
  const float c1 = tab.c1;
  const int nblk = two ? 2 : 1;
  uint4 pre[Tile<DK>::LOADS];

  for (int round0 = c.t_begin; round0 < c.t_end; round0 += kRoundKeys) {
    // tile (wave, j) of the round covers keys round0 + (j * kWaves + wave) * 32 ...
    int t_next = round0 + wave * 32;
    if (t_next < c.t_end) T.fetch(pre, khead, I.tok_stride, t_next, c.t_end, lane);
    for (int jt = 0; jt < kRoundTiles; ++jt) {
      const int widx = jt * kWaves + wave;
      const int t0 = round0 + widx * 32;
      uint32_t bits[2] = {0u, 0u};
      if (t0 < c.t_end) {
        T.stage(pre, tiles[wave], lane);
        t_next = t0 + kWaves * 32;
        if (jt + 1 < kRoundTiles && t_next < c.t_end) T.fetch(pre, khead, I.tok_stride, t_next, c.t_end, lane);
        __builtin_amdgcn_wave_barrier();
        floatx16 acc[2];
        T.compute(acc, tiles[wave], lane, two);
        __builtin_amdgcn_wave_barrier();
        auto classify = [&](float d, int nb, int key) {
          const int a = (int)floorf(d * c1);
          if (a > astar[nb]) {
            bits[nb] |= 1u << key;
          } else if (a == astar[nb]) {
            const int nl = 32 * nb + col;
            const int slot = atomicAdd(&ccnt[nl], 1);
            if (slot < kLocalCand) cbuf[nl][slot] = make_uint2(__float_as_uint(d), (uint32_t)(t0 + key));
          }
        };
        if (t0 + 32 <= c.t_end) {
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) {
            if (nb < nblk) {
#pragma unroll
              for (int r = 0; r < 16; ++r) classify(acc[nb][r], nb, key_of(r, hf));
            }
          }
        } else {
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) {
            if (nb < nblk) {
#pragma unroll
              for (int r = 0; r < 16; ++r)
                if (t0 + key_of(r, hf) < c.t_end) classify(acc[nb][r], nb, key_of(r, hf));
            }
          }
        }
      }
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        const uint32_t w = bits[nb] | __shfl_xor(bits[nb], 32, 64);
        if (lane < 32) mwords[32 * nb + lane][widx] = w;
      }
    }
    __syncthreads();
    // mask words of this round: row n, words round0/32 .. ; every row writes one contiguous run
    {
      const int w_first = round0 >> 5;
      const int n_words = min(kWaves * kRoundTiles, ((c.t_end - round0) + 31) >> 5);
      for (int i = tid; i < 64 * kWaves * kRoundTiles; i += kThreads) {
        const int nl = i / (kWaves * kRoundTiles), w = i % (kWaves * kRoundTiles);
        const int n = c.n0 + nl;
        if (n < tab.NQ && w < n_words) {
          const int s = n / tab.G, g = n % tab.G;
          const int r = s * tab.Hq + c.kvh * tab.G + g;
          tab.rowmask[I.mask_off + (long long)r * I.W + w_first + w] = mwords[nl][w];
        }
      }
    }
    // boundary candidates of this round -> the rows' global lists
    if (tid < 64) {
      const int n = c.n0 + tid;
      int cnt = ccnt[tid];
      cbase[tid] = -1;
      if (n < tab.NQ && cnt > 0) {
        const int s = n / tab.G, g = n % tab.G;
        const int grow = row_base + s * tab.Hq + c.kvh * tab.G + g;
        if (cnt > kLocalCand) {
          tab.info[grow].flag = 1;
        } else {
          const int b = atomicAdd(&tab.cand_cnt[grow], cnt);
          if (b + cnt <= kCandCap) cbase[tid] = b;   // otherwise resolve sees the count and flags the row
        }
      }
    }
    __syncthreads();
    for (int i = tid; i < 64 * kLocalCand; i += kThreads) {
      const int nl = i / kLocalCand, sl = i % kLocalCand;
      const int b = cbase[nl];
      if (b >= 0 && sl < ccnt[nl]) {
        const int n = c.n0 + nl;
        const int s = n / tab.G, g = n % tab.G;
        const int grow = row_base + s * tab.Hq + c.kvh * tab.G + g;
        tab.cands[(size_t)grow * kCandCap + b + sl] = cbuf[nl][sl];
      }
    }
    __syncthreads();
    if (tid < 64) ccnt[tid] = 0;
    __syncthreads();
  }
}

// ------------------------------------------------------------------ per row: exact cut among the candidates
__global__ __launch_bounds__(256) void resolve_kernel(const FastTable tab) {
  const int grow = blockIdx.x;
  RowInfo *info = tab.info + grow;
  const int tid = threadIdx.x;
  if (info->flag) return;
  const int cnt = tab.cand_cnt[grow];
  if (cnt > kCandCap) {
    if (tid == 0) info->flag = 1;
    return;
  }
  const int it = grow / tab.rows_per_item, r = grow - it * tab.rows_per_item;
  const FastItem I = tab.it[it];
  __shared__ unsigned long long key[kCandCap];
  __shared__ float wgt[kCandCap];
  __shared__ float hist[256];
  __shared__ int hcnt[256];
  __shared__ unsigned long long sh_prefix;
  __shared__ double sh_above;
  const float ref = info->mdot * tab.c2;
  const uint2 *src = tab.cands + (size_t)grow * kCandCap;
  for (int i = tid; i < cnt; i += 256) {
    const uint2 e = src[i];
    const float d = __uint_as_float(e.x);
    key[i] = ((unsigned long long)ordered_bits(d) << 32) | (unsigned long long)(0xFFFFFFFFu - e.y);
    wgt[i] = exp2f(fmaf(d, tab.c2, -ref));
  }
  if (tid == 0) { sh_prefix = 0ull; sh_above = info->above; }
  const double target = info->target;
  __syncthreads();
  for (int pass = 0; pass < 8; ++pass) {
    const int shift = 56 - 8 * pass;
    hist[tid] = 0.f;
    hcnt[tid] = 0;
    __syncthreads();
    const unsigned long long prefix = sh_prefix;
    for (int i = tid; i < cnt; i += 256) {
      const unsigned long long k = key[i];
      if (pass == 0 || (k >> (shift + 8)) == prefix) {
        const int dg = (int)((k >> shift) & 255ull);
        atomicAdd(&hist[dg], wgt[i]);
        atomicAdd(&hcnt[dg], 1);
      }
    }
    __syncthreads();
    if (tid < 64) {
      double above = sh_above;
      const int pick = pick_digit_wave(hist, hcnt, above, target, tid);
      if (tid == 0) {
        sh_prefix = (prefix << 8) | (unsigned long long)pick;
        sh_above = above;
      }
    }
    __syncthreads();
  }
  const unsigned long long tau = sh_prefix;
  uint32_t *mrow = tab.rowmask + I.mask_off + (long long)r * I.W;
  for (int i = tid; i < cnt; i += 256) {
    if (key[i] >= tau) {
      const uint32_t t = 0xFFFFFFFFu - (uint32_t)(key[i] & 0xFFFFFFFFull);
      atomicOr(&mrow[t >> 5], 1u << (t & 31));
    }
  }
}

int pick_chunk_keys(const gvote_shape *sh, const gvote_item *items, int n_items) {
  // about four workgroups per CU over the batch; a chunk is a whole number of emit rounds
  long long keys = 0;
  for (int i = 0; i < n_items; ++i) keys += (long long)items[i].L * sh->n_kv_heads;
  long long ck = (keys + 1023) / 1024;
  ck = (ck + kRoundKeys - 1) / kRoundKeys * kRoundKeys;
  if (ck < kRoundKeys) ck = kRoundKeys;
  if (ck > 8 * kRoundKeys) ck = 8 * kRoundKeys;
  return (int)ck;
}

}  // namespace

bool fast_path_ok(const gvote_shape *sh, int S, int mode, float p) {
  const int NQ = S * (sh->n_q_heads / sh->n_kv_heads);
  return sh->dtype == GVOTE_BF16 && (sh->head_dim == 64 || sh->head_dim == 128) && mode == GVOTE_SELECT_TOPP &&
         p < 1.0f && NQ >= 1;
}

FastPlan plan_fast(const gvote_shape *sh, const gvote_item *items, int n_items, int S) {
  FastPlan pl;
  const int NQ = S * (sh->n_q_heads / sh->n_kv_heads);
  size_t max_slots = 0, max_rows = 0;
  for (int b0 = 0; b0 < n_items; b0 += kMaxItems) {
    const int nb = n_items - b0 < kMaxItems ? n_items - b0 : kMaxItems;
    const int ck = pick_chunk_keys(sh, items + b0, nb);
    size_t slots = 0;
    for (int i = 0; i < nb; ++i) slots += (size_t)sh->n_kv_heads * ceil_div(items[b0 + i].L, ck);
    if (slots > max_slots) max_slots = slots;
    const size_t rows = (size_t)nb * S * sh->n_q_heads;
    if (rows > max_rows) max_rows = rows;
  }
  pl.off_max = 256;   // the first 256 bytes hold the fallback-row counter
  pl.off_hist = pl.off_max + align_up(max_slots * NQ * sizeof(float), 256);
  pl.off_info = pl.off_hist + align_up(max_slots * NQ * kBins * sizeof(float), 256);
  pl.off_cnt = pl.off_info + align_up(max_rows * sizeof(RowInfo), 256);
  pl.off_cands = pl.off_cnt + align_up(max_rows * sizeof(int), 256);
  pl.ws_bytes = pl.off_cands + align_up(max_rows * kCandCap * sizeof(uint2), 256);
  return pl;
}

gvote_status launch_score_fast(const gvote_shape *sh, const gvote_item *items, int n_items, int S, const void *q,
                               float p, uint32_t *rowmask, float *row_max, float *row_sum, void *ws, hipStream_t st) {
  const FastPlan pl = plan_fast(sh, items, n_items, S);
  char *wsb = reinterpret_cast<char *>(ws);
  const int G = sh->n_q_heads / sh->n_kv_heads;
  long long mask_off = 0;
  for (int b0 = 0; b0 < n_items; b0 += kMaxItems) {
    const int nb = n_items - b0 < kMaxItems ? n_items - b0 : kMaxItems;
    const long long batch_mask_off0 = mask_off;
    FastTable tab;
    tab.n_items = nb; tab.S = S; tab.Hq = sh->n_q_heads; tab.Hkv = sh->n_kv_heads; tab.G = G;
    tab.NQ = S * G; tab.NQB = (tab.NQ + 63) / 64;
    tab.chunk_keys = pick_chunk_keys(sh, items + b0, nb);
    tab.item0 = b0; tab.rows_per_item = S * sh->n_q_heads;
    tab.scale = (float)(1.0 / sqrt((double)sh->head_dim));
    tab.c1 = tab.scale * (float)kBinsPerUnit;
    tab.c2 = tab.scale * 1.44269504088896340736f;
    tab.p = p;
    tab.q = q; tab.rowmask = rowmask; tab.row_max = row_max; tab.row_sum = row_sum;
    tab.n_fallback = reinterpret_cast<int *>(wsb);
    tab.part_max = reinterpret_cast<float *>(wsb + pl.off_max);
    tab.part_hist = reinterpret_cast<float *>(wsb + pl.off_hist);
    tab.info = reinterpret_cast<RowInfo *>(wsb + pl.off_info);
    tab.cand_cnt = reinterpret_cast<int *>(wsb + pl.off_cnt);
    tab.cands = reinterpret_cast<uint2 *>(wsb + pl.off_cands);
    int wg = 0, part = 0;
    for (int i = 0; i < nb; ++i) {
      const gvote_item &g = items[b0 + i];
      FastItem &f = tab.it[i];
      f.k = g.k; f.tok_stride = g.kv_tok_stride; f.head_stride = g.kv_head_stride;
      f.mask_off = mask_off; f.L = g.L; f.W = (g.L + 31) / 32;
      f.n_chunks = ceil_div(g.L, tab.chunk_keys);
      f.wg0 = wg; f.part0 = part; f.pad = 0;
      wg += sh->n_kv_heads * f.n_chunks * tab.NQB;
      part += sh->n_kv_heads * f.n_chunks;
      mask_off += (long long)tab.rows_per_item * f.W;
    }
    const int rows = nb * tab.rows_per_item;
    if (sh->head_dim == 128) {
      hipLaunchKernelGGL(score_max_kernel<128>, dim3(wg), dim3(kThreads), 0, st, tab);
      GVOTE_CHECK_LAUNCH();
      hipLaunchKernelGGL(score_hist_kernel<128>, dim3(wg), dim3(kThreads), 0, st, tab);
      GVOTE_CHECK_LAUNCH();
      hipLaunchKernelGGL(find_bin_kernel, dim3(rows), dim3(kBins), 0, st, tab);
      GVOTE_CHECK_LAUNCH();
      hipLaunchKernelGGL(score_emit_kernel<128>, dim3(wg), dim3(kThreads), 0, st, tab);
    } else {
      hipLaunchKernelGGL(score_max_kernel<64>, dim3(wg), dim3(kThreads), 0, st, tab);
      GVOTE_CHECK_LAUNCH();
      hipLaunchKernelGGL(score_hist_kernel<64>, dim3(wg), dim3(kThreads), 0, st, tab);
      GVOTE_CHECK_LAUNCH();
      hipLaunchKernelGGL(find_bin_kernel, dim3(rows), dim3(kBins), 0, st, tab);
      GVOTE_CHECK_LAUNCH();
      hipLaunchKernelGGL(score_emit_kernel<64>, dim3(wg), dim3(kThreads), 0, st, tab);
    }
    GVOTE_CHECK_LAUNCH();
    hipLaunchKernelGGL(resolve_kernel, dim3(rows), dim3(256), 0, st, tab);
    GVOTE_CHECK_LAUNCH();
    // rows the histogram could not settle are redone exactly
    gvote_status stt = launch_select_rows_general(sh, items + b0, nb, b0, S, q, p, GVOTE_SELECT_TOPP, nullptr, rowmask,
                                                  batch_mask_off0, row_max, row_sum, &tab.info[0].flag,
                                                  (int)(sizeof(RowInfo) / sizeof(int)), tab.n_fallback, st);
    if (stt != GVOTE_OK) return stt;
  }
  return GVOTE_OK;
}

}  // namespace gvote
