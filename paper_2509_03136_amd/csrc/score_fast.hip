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
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));   // one 16-byte lane of a K row

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

// Fixed-point histogram bins (integer LDS atomics run ~30x faster than float ones on this chip).
// Bins live on an absolute grid of the raw dot product d: a = floor(d * c1), 16 bins per unit of
// logit.  A key adds exp((l - E_a)) * 2^kFixBits to its bin, E_a the bin's UPPER edge, so every term
// lies in (0.94, 1] * 2^18 whatever the row maximum is, and a chunk of <= 8192 keys cannot overflow
// 32 bits.  Bin j of a row is absolute bin top - j (top = bin of the row maximum); everything deeper
// than kBins - 1 bins is clamped into the last bin, measured against that bin's edge (such keys weigh
// < 1.2e-7 of the maximum each; below 2^-19 of the edge they round to nothing).
constexpr int kFixBits = 18;
constexpr float kLog2ePerBin = 1.44269504088896340736f / (float)kBinsPerUnit;   // log2 weight per bin

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

  // coalesced fetch of keys t0 .. t0+31 of one KV head.  No branches (the compiler then counts the
  // outstanding loads exactly and the two-tile prefetch really overlaps): positions at or beyond `end`
  // re-read key end-1, their products are discarded by the caller's validity test.
  __device__ __forceinline__ void fetch(u32x4 (&pre)[LOADS], const bf16_t *khead, long long tok_stride, int t0, int end,
                                        int lane) const {
    const int piece = lane % PPR, sub = lane / PPR;
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
      const int t = min(t0 + j * RPL + sub, end - 1);
      pre[j] = *reinterpret_cast<const u32x4 *>(khead + (long long)t * tok_stride + piece * 8);
    }
  }

  __device__ __forceinline__ void stage(const u32x4 (&pre)[LOADS], unsigned char *lds, int lane) const {
    const int piece = lane % PPR, sub = lane / PPR;
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
      const int key = j * RPL + sub;
      const int phys = piece ^ (key & (PPR - 1));
      *reinterpret_cast<u32x4 *>(lds + (key * PPR + phys) * 16) = pre[j];
    }
  }

  // all eight A operands are read before the first MFMA so the LDS latency is paid once per tile
  template <bool TWO>
  __device__ __forceinline__ void compute(floatx16 (&acc)[2], const unsigned char *lds, int lane) const {
    const int key = lane & 31, hf = lane >> 5;
    bf16x8 a[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      const int phys = (2 * ks + hf) ^ (key & (PPR - 1));
      a[ks] = *reinterpret_cast<const bf16x8 *>(lds + (key * PPR + phys) * 16);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc[0][r] = 0.f; acc[1][r] = 0.f; }
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], bq[0][ks], acc[0], 0, 0, 0);
      if (TWO) acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[ks], bq[1][ks], acc[1], 0, 0, 0);
    }
  }
};

// The K stream of one wave: tiles wave, wave + 8, wave + 16, ... of the chunk [t_begin, t_end), with the
// global loads of the next TWO tiles in flight (registers) while the current one is multiplied: with
// 8 waves per CU that keeps 128 KiB per CU outstanding, what HBM latency needs at full bandwidth.
// `epi(acc, t0)` consumes a tile's 32 x 64 products; `round_end(round)` runs after every kRoundTiles
// tiles of every wave (all waves call it equally often, so it may hold workgroup barriers).
template <int DK, bool TWO, class Epi, class RoundEnd>
__device__ __forceinline__ void stream_tiles_impl(const Tile<DK> &T, unsigned char *lds, const bf16_t *khead,
                                                  long long tok_stride, int t_begin, int t_end, int wave, int lane,
                                                  Epi &&epi, RoundEnd &&round_end) {
  constexpr int LOADS = Tile<DK>::LOADS;
  const int n_tiles = (t_end - t_begin + 31) >> 5;
  const int n_rounds = (n_tiles + kWaves * kRoundTiles - 1) / (kWaves * kRoundTiles);
  u32x4 pa[LOADS], pb[LOADS];
  // (positions are clamped inside fetch, so the first two fetches need no guard)
  T.fetch(pa, khead, tok_stride, t_begin + wave * 32, t_end, lane);
  T.fetch(pb, khead, tok_stride, t_begin + (wave + kWaves) * 32, t_end, lane);
  for (int k = 0; k < n_rounds * kRoundTiles; k += 2) {
    {
      const int tile = wave + kWaves * k;
      if (tile < n_tiles) {
        const int t0 = t_begin + tile * 32;
        T.stage(pa, lds, lane);
        if (tile + 2 * kWaves < n_tiles) T.fetch(pa, khead, tok_stride, t0 + 2 * kWaves * 32, t_end, lane);
        __builtin_amdgcn_wave_barrier();
        floatx16 acc[2];
        T.template compute<TWO>(acc, lds, lane);
        __builtin_amdgcn_wave_barrier();
        epi(acc, t0, k);
      }
    }
    {
      const int tile = wave + kWaves * (k + 1);
      if (tile < n_tiles) {
        const int t0 = t_begin + tile * 32;
        T.stage(pb, lds, lane);
        if (tile + 2 * kWaves < n_tiles) T.fetch(pb, khead, tok_stride, t0 + 2 * kWaves * 32, t_end, lane);
        __builtin_amdgcn_wave_barrier();
        floatx16 acc[2];
        T.template compute<TWO>(acc, lds, lane);
        __builtin_amdgcn_wave_barrier();
        epi(acc, t0, k + 1);
      }
    }
    if ((k + 2) % kRoundTiles == 0) round_end((k + 2) / kRoundTiles - 1);
  }
}

template <int DK, class Epi, class RoundEnd>
__device__ __forceinline__ void stream_tiles(const Tile<DK> &T, unsigned char *lds, const bf16_t *khead,
                                             long long tok_stride, int t_begin, int t_end, int wave, int lane,
                                             bool two, Epi &&epi, RoundEnd &&round_end) {
  if (two)
    stream_tiles_impl<DK, true>(T, lds, khead, tok_stride, t_begin, t_end, wave, lane, epi, round_end);
  else
    stream_tiles_impl<DK, false>(T, lds, khead, tok_stride, t_begin, t_end, wave, lane, epi, round_end);
}

// ------------------------------------------------------------------ pass A: chunk maxima
template <int DK>
__global__ __launch_bounds__(kThreads) void score_max_kernel(const FastTable tab) {
  __shared__ __align__(16) unsigned char tiles[kWaves][Tile<DK>::BYTES];
  __shared__ uint32_t smax[64];
  const WgCoord c = decode_wg(tab, blockIdx.x);
  const FastItem I = tab.it[c.it];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hf = lane >> 5;
  if (tid < 64) smax[tid] = 0u;
  Tile<DK> T;
  T.load_q(tab, c.it, c.kvh, c.n0, lane);
  const bool two = c.n0 + 32 < tab.NQ;
  const bf16_t *khead = reinterpret_cast<const bf16_t *>(I.k) + (long long)c.kvh * I.head_stride;
  float mx[2] = {-INFINITY, -INFINITY};
  __syncthreads();
  stream_tiles<DK>(
      T, tiles[wave], khead, I.tok_stride, c.t_begin, c.t_end, wave, lane, two,
      [&](const floatx16(&acc)[2], int t0, int) __attribute__((always_inline)) {
        if (t0 + 32 <= c.t_end) {
#pragma unroll
          for (int r = 0; r < 16; ++r) { mx[0] = fmaxf(mx[0], acc[0][r]); mx[1] = fmaxf(mx[1], acc[1][r]); }
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            if (t0 + key_of(r, hf) < c.t_end) { mx[0] = fmaxf(mx[0], acc[0][r]); mx[1] = fmaxf(mx[1], acc[1][r]); }
          }
        }
      },
      [](int) {});
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
  __shared__ uint32_t hist[64 * (kBins + 1)];
  __shared__ int s_top[64];
  const WgCoord c = decode_wg(tab, blockIdx.x);
  const FastItem I = tab.it[c.it];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hf = lane >> 5, col = lane & 31;
  for (int i = tid; i < 64 * (kBins + 1); i += kThreads) hist[i] = 0u;
  if (tid < 64) {
    float m = -INFINITY;
    if (c.n0 + tid < tab.NQ) {
      const float *pm = tab.part_max + (size_t)(I.part0 + c.kvh * I.n_chunks) * tab.NQ + c.n0 + tid;
      for (int ch = 0; ch < I.n_chunks; ++ch) m = fmaxf(m, pm[(size_t)ch * tab.NQ]);
    }
    s_top[tid] = (int)floorf(m * tab.c1);
  }
  Tile<DK> T;
  T.load_q(tab, c.it, c.kvh, c.n0, lane);
  const bool two = c.n0 + 32 < tab.NQ;
  const bf16_t *khead = reinterpret_cast<const bf16_t *>(I.k) + (long long)c.kvh * I.head_stride;
  __syncthreads();
  const int nblk = two ? 2 : 1;
  int top[2];
  uint32_t *hrow[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    top[nb] = s_top[32 * nb + col];
    hrow[nb] = hist + (32 * nb + col) * (kBins + 1);
  }
  const float c1 = tab.c1, c2 = tab.c2;
  // x = d * c2 - (a + 1) * kLog2ePerBin + kFixBits is log2 of the fixed-point term of a key in bin a
  const float ebias = (float)kFixBits - kLog2ePerBin;
  float atail[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    if (c.n0 + 32 * nb + col >= tab.NQ) top[nb] = 1 << 24;   // rows that do not exist: always the last bin, weight 0
    atail[nb] = (float)(top[nb] - (kBins - 1));
  }
  stream_tiles<DK>(
      T, tiles[wave], khead, I.tok_stride, c.t_begin, c.t_end, wave, lane, two,
      [&](const floatx16(&acc)[2], int t0, int) __attribute__((always_inline)) {
        const bool full = t0 + 32 <= c.t_end;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          if (nb < nblk) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
              const float d = acc[nb][r];
              const float af = fmaxf(floorf(d * c1), atail[nb]);
              const float x = fmaf(d, c2, fmaf(af, -kLog2ePerBin, ebias));
              uint32_t u = (uint32_t)(__builtin_amdgcn_exp2f(x) + 0.5f);
              if (!full) u = t0 + key_of(r, hf) < c.t_end ? u : 0u;
              atomicAdd(hrow[nb] + (top[nb] - (int)af), u);
            }
          }
        }
      },
      [](int) {});
  __syncthreads();
  uint32_t *out = tab.part_hist + ((size_t)c.slot * tab.NQ + c.n0) * kBins;
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
  float m = -INFINITY;
  for (int ch = 0; ch < I.n_chunks; ++ch) m = fmaxf(m, tab.part_max[(slot0 + ch) * tab.NQ + n]);
  unsigned long long acc = 0ull;
  for (int ch = 0; ch < I.n_chunks; ++ch) acc += tab.part_hist[((slot0 + ch) * tab.NQ + n) * kBins + j];
  // weight of bin j relative to exp(max): fixed-point sum * 2^-kFixBits * exp2(edge_j - max), in log2 units
  const int top = (int)floorf(m * tab.c1);
  const double edge = (double)(top - j + 1) * (double)kLog2ePerBin;
  const double mine = ldexp((double)acc, -kFixBits) * exp2(edge - (double)m * (double)tab.c2);
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
  __shared__ int s_row[64];      // row index (s * H_q + h) of the workgroup's 64 query rows, -1 if absent
  const WgCoord c = decode_wg(tab, blockIdx.x);
  const FastItem I = tab.it[c.it];
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hf = lane >> 5, col = lane & 31;
  const int row_base = c.it * tab.rows_per_item;   // batch-local row index of (s = 0, h = 0)
  if (tid < 64) {
    const int n = c.n0 + tid;
    int a = 0x7FFFFFFF, r = -1;
    if (n < tab.NQ) {
      const int s = n / tab.G, g = n % tab.G;
      r = s * tab.Hq + c.kvh * tab.G + g;
      a = tab.info[row_base + r].astar;
    }
    s_astar[tid] = a;
    s_row[tid] = r;
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
  constexpr int kRoundWords = kWaves * kRoundTiles;
  // raw dot below which a key surely lies under the row's cut bin (half a bin of margin; rows that do
  // not exist carry astar = INT_MAX and never match)
  float dcut[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) dcut[nb] = astar[nb] == 0x7FFFFFFF ? INFINITY : ((float)astar[nb] - 0.5f) / c1;

  stream_tiles<DK>(
      T, tiles[wave], khead, I.tok_stride, c.t_begin, c.t_end, wave, lane, two,
      [&](const floatx16(&acc)[2], int t0, int k) __attribute__((always_inline)) {
        uint32_t bits[2] = {0u, 0u};
        const bool full = t0 + 32 <= c.t_end;
        // most tiles hold no key at or above any row's cut bin: one max per row settles that
        float mx0 = acc[0][0], mx1 = acc[1][0];
#pragma unroll
        for (int r = 1; r < 16; ++r) { mx0 = fmaxf(mx0, acc[0][r]); mx1 = fmaxf(mx1, acc[1][r]); }
        const bool near = mx0 >= dcut[0] || mx1 >= dcut[1];
        if (__any(near)) {
          uint32_t cmask[2] = {0u, 0u};
#pragma unroll
          for (int nb = 0; nb < 2; ++nb) {
            if (nb < nblk) {
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                const int key = key_of(r, hf);
                const bool valid = full || t0 + key < c.t_end;
                const int a = (int)floorf(acc[nb][r] * c1);
                bits[nb] |= (valid && a > astar[nb]) ? (1u << key) : 0u;
                cmask[nb] |= (valid && a == astar[nb]) ? (1u << r) : 0u;
              }
            }
          }
          if (__any((cmask[0] | cmask[1]) != 0u)) {   // keys inside the cut bin: rare
#pragma unroll
            for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
              for (int r = 0; r < 16; ++r) {
                if (cmask[nb] & (1u << r)) {
                  const int nl = 32 * nb + col;
                  const int slot = atomicAdd(&ccnt[nl], 1);
                  if (slot < kLocalCand)
                    cbuf[nl][slot] = make_uint2(__float_as_uint(acc[nb][r]), (uint32_t)(t0 + key_of(r, hf)));
                }
              }
            }
          }
        }
        const int widx = (k % kRoundTiles) * kWaves + wave;
#pragma unroll
        for (int nb = 0; nb < 2; ++nb) {
          const uint32_t w = bits[nb] | __shfl_xor(bits[nb], 32, 64);
          if (lane < 32) mwords[32 * nb + lane][widx] = w;
        }
      },
      [&](int round) __attribute__((always_inline)) {
        const int round0 = c.t_begin + round * kRoundKeys;
        __syncthreads();
        // mask words of this round: every row writes one contiguous run of up to 128 bytes
        const int w_first = round0 >> 5;
        const int n_words = min(kRoundWords, ((c.t_end - round0) + 31) >> 5);
        for (int i = tid; i < 64 * kRoundWords; i += kThreads) {
          const int nl = i / kRoundWords, w = i % kRoundWords;
          const int r = s_row[nl];
          if (r >= 0 && w < n_words) tab.rowmask[I.mask_off + (long long)r * I.W + w_first + w] = mwords[nl][w];
        }
        // boundary candidates of this round -> the rows' global lists
        if (tid < 64) {
          const int cnt = ccnt[tid];
          const int r = s_row[tid];
          cbase[tid] = -1;
          if (r >= 0 && cnt > 0) {
            if (cnt > kLocalCand) {
              tab.info[row_base + r].flag = 1;
            } else {
              const int b = atomicAdd(&tab.cand_cnt[row_base + r], cnt);
              if (b + cnt <= kCandCap) cbase[tid] = b;   // else resolve sees the count and flags the row
            }
          }
        }
        __syncthreads();
        for (int i = tid; i < 64 * kLocalCand; i += kThreads) {
          const int nl = i / kLocalCand, sl = i % kLocalCand;
          const int b = cbase[nl];
          if (b >= 0 && sl < ccnt[nl]) tab.cands[(size_t)(row_base + s_row[nl]) * kCandCap + b + sl] = cbuf[nl][sl];
        }
        __syncthreads();
        if (tid < 64) ccnt[tid] = 0;
        __syncthreads();
      });
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
    tab.part_hist = reinterpret_cast<uint32_t *>(wsb + pl.off_hist);
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
