// Stage 3, bf16 fast path - K-streaming scores on the matrix cores and a histogram search for the
// mass-p cut (paper Eq. (1) logits and softmax weights; Sec. 3.1 minimal key set of mass p).  Alg. 1's
// row-wise TopK on logits is the same search with unit weights (bins hold key counts, the target is k).
//
// Nothing of size S*H_q*L is stored: logits are recomputed from K in each pass, bit-identically
// (same MFMA sequence), and only per-row statistics travel between the passes.
//
//   score_hist   pass 1 over K: per (item, KV head, key chunk) the row maxima and, in LDS, a 256-bin
//                fixed-point histogram per query row of the weight exp(l) on an absolute grid of
//                1/16 logit; the window of bins slides up with the running maximum.  Also leaves the
//                per (32-key tile, row) maxima.
//   find_bin     per row: merge the chunks, Z, target p*Z, walk the bins from the top: the bin
//                a* where the cumulative weight crosses the target, and the weight above it.
//   score_refine a second histogram for the rows the first cannot settle (does nothing otherwise): a
//   refine_bin   cut below the window gets a window right below it; a cut bin with more keys than
//                pass 2 can list is split into 256 bins of 1/4096 logit.  Same grid arithmetic, the
//                window top is fixed, keys above it are ignored.
//   score_emit   pass 2 over K, only over tiles whose maxima reach some row's cut bin: keys in bins
//                above a* are selected outright (bit masks, transposed in LDS so every row writes
//                whole 128-byte runs); keys inside bin a* are appended (raw dot, position) to the
//                row's candidate list.
//   resolve      per row (one wave): exact selection among the candidates in the order (raw dot
//                descending, position ascending), so ties go to the lower position - a pairwise
//                "weight ahead of me" test for up to 64 candidates, a radix search beyond - and OR
//                of the chosen bits into the mask.
// Rows whose cut falls below the second window as well, or whose candidate lists still overflow, are
// queued and redone by the exact general selector (select_row_kernel).
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
// lies in (0.94, 1] * 2^17 whatever the row maximum is, and a chunk of <= 16384 keys cannot overflow
// 32 bits.  Bin j of a row is absolute bin top - j (top = bin of the row maximum); everything deeper
// than kBins - 1 bins is clamped into the last bin, measured against that bin's edge (such keys weigh
// < 1.2e-7 of the maximum each; below 2^-19 of the edge they round to nothing).
constexpr int kFixBits = 17;
constexpr float kLog2ePerBin = 1.44269504088896340736f / (float)kBinsPerUnit;   // log2 weight per bin

// integer add to a 32-bit word of LDS given its byte address inside the workgroup's LDS
typedef __attribute__((address_space(3))) uint32_t lds_u32;
__device__ __forceinline__ void lds_add_u32(uint32_t byte_addr, uint32_t v) {
#if defined(__HIP_DEVICE_COMPILE__)
  __hip_atomic_fetch_add((lds_u32 *)(size_t)byte_addr, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
#else
  (void)byte_addr; (void)v;
#endif
}
typedef __attribute__((address_space(3))) int lds_int;    // (workgroup flags are polled with LDS loads: a generic-
                                                          // pointer load would also wait for every global load in flight)
// byte offset of an LDS object inside the workgroup's LDS
__device__ __forceinline__ int lds_offset(const void *p) {
#if defined(__HIP_DEVICE_COMPILE__)
  return (int)(size_t)(const __attribute__((address_space(3))) char *)p;
#else
  (void)p; return 0;
#endif
}

// A tile nominally covers keys t0 .. t0+31 of the chunk ending at `end`; when that would run past the
// end the 32 keys end-32 .. end-1 are loaded instead (every item has at least 32 keys) and the first
// t0 - origin of them, which belong to the previous tile or chunk, are ignored.
__device__ __forceinline__ int tile_origin(int t0, int end) { return min(t0, end - 32); }

// Bin number of a scaled dot for the window logic.  Bin numbers are kept inside +-2^20 (65536 logit units) whatever
// the data holds (huge values, infinities, NaN -> the lower limit): LDS addresses are formed as 4 * bin + offset in
// fp32, which is exact only for small integers, and an address outside the workgroup's LDS must never be issued.
constexpr float kBinLimit = 1048576.0f;
__device__ __forceinline__ int bin_of(float y) { return (int)fminf(fmaxf(floorf(y), -kBinLimit), kBinLimit); }

// position of accumulator register r of lane (hf = lane / 32) inside the 32-key tile
__device__ __forceinline__ int key_of(int r, int hf) { return 8 * (r >> 2) + 4 * hf + (r & 3); }

struct WgCoord {
  int it, kvh, chunk, qb, n0, t_begin, t_end, slot;
};

// Workgroup ids go round-robin over the 8 XCDs (each with its own L2).  When a KV group has more than
// 64 query rows, its NQB row blocks all stream the same keys: the launch order is permuted so that the
// NQB workgroups of one (head, chunk) slot get ids 8 apart, i.e. land on the same XCD close in time and
// share the chunk through that XCD's L2.  Returns false for the padding ids of the last group.
__device__ __forceinline__ bool xcd_order(const FastTable &tab, int &wg) {
  if (tab.NQB == 1) return true;
  const int per = 8 * tab.NQB;
  const int group = wg / per, within = wg - group * per;
  const int qb = within >> 3, slot = group * 8 + (within & 7);
  if (slot >= tab.n_slots) return false;
  wg = slot * tab.NQB + qb;
  return true;
}

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

// NT: the keys are read once by this workgroup and by nobody else soon (one block of 64 rows per KV head): non-temporal
// loads keep them from displacing anything (+7 % on pass 1).  With several row blocks per KV head the blocks of one
// chunk run side by side on one XCD and share its L2: ordinary loads then (pass 2 -24 % at 224 rows per KV head).
template <int DK, bool NT>
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

  // Coalesced fetch of the 32 keys t .. t+31 of one KV head, all of which must exist (callers pull a
  // ragged last tile back to `end - 32`, see tile_origin).  Addresses are (wave-uniform base) + (32-bit
  // lane offset) and nothing is conditional, so the loads of several tiles stay in flight together.
  __device__ __forceinline__ void fetch(u32x4 (&pre)[LOADS], const bf16_t *khead, long long tok_stride, int t,
                                        int lane) const {
    const int piece = lane % PPR, sub = lane / PPR;
    const char *tile = reinterpret_cast<const char *>(khead) + (long long)t * tok_stride * 2;
    const uint32_t lane_off = (uint32_t)(sub * (int)tok_stride + piece * 8) * 2u;
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
      const char *src = tile + (long long)(j * RPL) * tok_stride * 2 + lane_off;
      pre[j] = NT ? load_stream16(src) : *reinterpret_cast<const u32x4 *>(src);
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

  // the A operands are read four k-steps at a time ahead of their MFMAs: the LDS latency is paid twice
  // per tile and only 16 registers hold operands
  template <bool TWO>
  __device__ __forceinline__ void compute(floatx16 (&acc)[2], const unsigned char *lds, int lane) const {
    const int key = lane & 31, hf = lane >> 5;
#pragma unroll
    for (int r = 0; r < 16; ++r) { acc[0][r] = 0.f; acc[1][r] = 0.f; }
    constexpr int GRP = KS < 4 ? KS : 4;
#pragma unroll
    for (int k0 = 0; k0 < KS; k0 += GRP) {
      bf16x8 a[GRP];
#pragma unroll
      for (int i = 0; i < GRP; ++i) {
        const int phys = (2 * (k0 + i) + hf) ^ (key & (PPR - 1));
        a[i] = *reinterpret_cast<const bf16x8 *>(lds + (key * PPR + phys) * 16);
      }
#pragma unroll
      for (int i = 0; i < GRP; ++i) {
        acc[0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bq[0][k0 + i], acc[0], 0, 0, 0);
        if (TWO) acc[1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], bq[1][k0 + i], acc[1], 0, 0, 0);
      }
    }
  }
};

// ------------------------------------------------------------------ pass 1: maxima + weight histograms, one K read
// The row maximum is not known while the chunk streams by, so the 256-bin window of each row slides:
// bins sit on the absolute grid a = floor(d * c1) and hold weights relative to their own upper edge,
// hence raising a window is a plain shift of the LDS row (bins pushed past the end are re-referenced
// into the last bin).  Waves run free of each other; only when a wave meets a key above a window top
// (after the first tile: rarely, tops carry two units of headroom) does it call for a workgroup event:
//   requester: record the new maximum, set `pending`, enter the event;
//   every wave looks at `pending` before it bins a tile (and while it idles after its last tile), so all
//   eight waves enter the same event exactly once: barrier - each wave slides the windows of the eight
//   rows it owns - `pending` cleared - barrier - reload the tops.
// Inside an event no wave touches the histogram, outside nobody moves it.  A wave that has finished its
// tiles keeps serving events until all eight have finished (`done`).
struct HistCtl {
  int top[64];          // window top (absolute bin) of each row, kTopUnset before the first key
  uint32_t newmax[64];  // ordered bits of the largest raw dot that asked for a higher window
  uint32_t rowmax[64];  // ordered bits of the chunk maximum of each row
  int pending, done, aborted, pad;
};
constexpr int kTopUnset = -(1 << 24);
constexpr int kTopGaveUp = -(1 << 25);   // part_top of a (slot, row) whose pass-1 workgroup gave up: find_bin sends the row to the exact selector
constexpr int kHeadroom = 4 * kBinsPerUnit;
constexpr int kFineShift = 8, kFineBins = 1 << kFineShift;   // bins inside a cut bin: 1/4096 of a logit unit
constexpr int kFineSpan = 1 << 13;     // |bin| below which fine bin numbers (x 256, x 4 bytes) stay exact in the fp32 address arithmetic: 512 logit units
constexpr int kFineTrigger = 3500;     // keys in a cut bin beyond which it is looked into (the resolver holds kCandCap = 4096)
constexpr int kRefineLevels = 1;        // further 256-bin windows below the first for rows whose cut lies deeper (one more
                                        // reaches 28..32 units below the maximum: weights of e^-28, beyond what fp32 sums resolve;
                                        // each level costs two launches that do nothing in the usual case)

template <int DK, bool TWO, bool TOPK, bool NT>
__device__ __forceinline__ void hist_fused_body(const FastTable &tab, const WgCoord &c, const FastItem &I,
                                                unsigned char *ldstile, uint32_t *hist, HistCtl *S) {
  constexpr int LOADS = Tile<DK, true>::LOADS;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hf = lane >> 5,
            col = lane & 31;
  Tile<DK, NT> T;
  T.load_q(tab, c.it, c.kvh, c.n0, lane);
  const bf16_t *khead = reinterpret_cast<const bf16_t *>(I.k) + (long long)c.kvh * I.head_stride;
  const int n_tiles = (c.t_end - c.t_begin + 31) >> 5;
  const int last_tile = wave < n_tiles ? wave + kWaves * ((n_tiles - 1 - wave) / kWaves) : n_tiles - 1;
  const float c1 = tab.c1, c2 = tab.c2;
  const float ebias = (float)kFixBits - kLog2ePerBin;
  uint32_t *hrow[2] = {hist + col * (kBins + 1), hist + (32 + col) * (kBins + 1)};
  volatile lds_int *pending = (volatile lds_int *)(size_t)lds_offset(&S->pending);
  volatile lds_int *done = (volatile lds_int *)(size_t)lds_offset(&S->done);
  int top[2] = {kTopUnset, kTopUnset};      // this lane's copy of its two rows' window tops
  float mxrun[2] = {-INFINITY, -INFINITY};

  auto sync_event = [&]() __attribute__((always_inline)) {
    __syncthreads();
    for (int rr = 0; rr < 8; ++rr) {
      const int row = 8 * wave + rr;
      const int amax = bin_of(from_ordered_bits(S->newmax[row]) * c1);
      const int oldtop = S->top[row];
      if (amax > oldtop) {            // wave-uniform
        const int newtop = amax + kHeadroom;
        uint32_t *h = hist + row * (kBins + 1);
        const long long sh = (long long)newtop - (long long)oldtop;
        constexpr int BPL = kBins / 64;     // bins per lane
        uint32_t v[BPL];
        float spill = 0.f;            // weight pushed past the window, re-referenced to the last bin's edge
#pragma unroll
        for (int i = 0; i < BPL; ++i) {
          const int j = lane * BPL + i;
          v[i] = h[j];
          const long long jn = j + sh;
          if (jn >= kBins - 1 && v[i] != 0u)
            spill += TOPK ? (float)v[i] : (float)v[i] * __builtin_amdgcn_exp2f(-(float)(jn - (kBins - 1)) * kLog2ePerBin);
        }
        for (int off = 32; off > 0; off >>= 1) spill += __shfl_xor(spill, off, 64);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int i = 0; i < BPL; ++i) {
          const int j = lane * BPL + i;       // destination bin
          const long long src = j - sh;
          // all lanes take part in the exchange (a lane must be active to be read from)
          // bin src lives in lane src / BPL at index src % BPL = (i - sh) mod BPL: the same index in every
          // lane, so each lane offers that element and the reader only chooses the lane
          const int sl = src >= 0 ? (int)(src / BPL) : 0;
          const int si = (int)((((long long)i - sh) % BPL + BPL) % BPL);
          uint32_t pick = v[0];
#pragma unroll
          for (int q = 1; q < BPL; ++q) pick = si == q ? v[q] : pick;
          const uint32_t got = __shfl(pick, sl, 64);
          h[j] = j == kBins - 1 ? (uint32_t)(spill + 0.5f) : (src >= 0 ? got : 0u);
        }
        if (lane == 0) S->top[row] = newtop;
      }
    }
    if (lane == 0) *pending = 0;      // between the barriers: nobody can be asking right now (every wave writes it:
                                      // no single wave's presence is needed, a wave may have given up and left)
    __syncthreads();
    top[0] = S->top[col];
    top[1] = S->top[32 + col];
  };

  auto tile_body = [&](u32x4(&pre)[LOADS], int tile) __attribute__((always_inline)) {
    const int t0 = c.t_begin + tile * 32;
    const int skip = t0 - tile_origin(t0, c.t_end);      // leading keys of the loaded window that are not this tile's
    floatx16 acc[2];
    // looked at early so the LDS latency hides behind the MFMAs; an event that opens after this look is
    // joined at the next tile (its barrier waits for this wave, so the histogram stays put meanwhile)
    const int pend_seen = *pending;
    T.stage(pre, ldstile, lane);
    {   // next tile of this wave (the last one is simply fetched again: no conditional load)
      const int tn = c.t_begin + min(tile + kWaves, last_tile) * 32;
      T.fetch(pre, khead, I.tok_stride, tile_origin(tn, c.t_end), lane);
    }
    __builtin_amdgcn_wave_barrier();
    T.template compute<TWO>(acc, ldstile, lane);
    __builtin_amdgcn_wave_barrier();
    // (keys ahead of a pulled-back tile are keys of the same row: they may enter the maxima, never the bins)
    float mx0 = acc[0][0], mx1 = acc[1][0];
#pragma unroll
    for (int r = 1; r < 16; ++r) { mx0 = fmaxf(mx0, acc[0][r]); mx1 = fmaxf(mx1, acc[1][r]); }
    mx0 = fmaxf(mx0, __shfl_xor(mx0, 32, 64));
    mx1 = fmaxf(mx1, __shfl_xor(mx1, 32, 64));
    mxrun[0] = fmaxf(mxrun[0], mx0);
    mxrun[1] = fmaxf(mxrun[1], mx1);
    const int amx0 = bin_of(mx0 * c1), amx1 = TWO ? bin_of(mx1 * c1) : 0;
    if (lane < 32) {        // bin of the largest dot of every (tile, row): pass 2 skips tiles no row needs
      short *tm = tab.tile_bin + I.tmax0 + ((size_t)c.kvh * I.W + (c.t_begin >> 5) + tile) * tab.NQ + c.n0 + col;
      if (c.n0 + col < tab.NQ) tm[0] = (short)max(-32768, min(32767, amx0));      // (saturated: pass 2 caps its side of the test at 32767, so saturation only ever keeps a tile)
      if (TWO && c.n0 + 32 + col < tab.NQ) tm[32] = (short)max(-32768, min(32767, amx1));
    }
    const bool over0 = amx0 > top[0];
    const bool over1 = TWO && amx1 > top[1];
    bool event = __any(over0 || over1);          // wave-uniform
    if (event) {
      if (lane < 32) {
        if (over0) atomicMax(&S->newmax[col], ordered_bits(mx0));
        if (over1) atomicMax(&S->newmax[32 + col], ordered_bits(mx1));
      }
      if (lane == 0) *pending = 1;
    } else {
      event = __builtin_amdgcn_readfirstlane(pend_seen) != 0;
    }
    if (event) sync_event();
    // Bin of a key: a = max(floor(d c1), top - 255); fixed-point term 2^(d c2 - (a + 1) log2e/16 + 17),
    // truncated (a uniform -2e-6 relative bias that cancels in every ratio of sums); LDS byte address
    // hrow + 4 (top - a), formed in fp32 (exact: all quantities are small integers).
    if (skip == 0) {
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        if (nb == 0 || TWO) {
          const float atail = (float)(top[nb] - (kBins - 1)), atop = (float)top[nb];
          const float abase = (float)(lds_offset(hrow[nb]) + 4 * top[nb]);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float d = acc[nb][r];
            const float af = __builtin_amdgcn_fmed3f(floorf(d * c1), atail, atop);     // (never above the top once the window has been raised: the upper clamp only keeps the address inside the row whatever the data)
            uint32_t u = 1u;        // TOPK counts keys
            if (!TOPK) u = (uint32_t)__builtin_amdgcn_exp2f(fmaf(d, c2, fmaf(af, -kLog2ePerBin, ebias)));
            lds_add_u32((uint32_t)fmaf(af, -4.0f, abase), u);
            if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);   // bounds the scheduler's look-ahead (registers)
          }
        }
      }
    } else {
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
        if (nb == 0 || TWO) {
          const float atail = (float)(top[nb] - (kBins - 1)), atop = (float)top[nb];
          const float abase = (float)(lds_offset(hrow[nb]) + 4 * top[nb]);
#pragma unroll
          for (int r = 0; r < 16; ++r) {
            const float d = acc[nb][r];
            const float af = __builtin_amdgcn_fmed3f(floorf(d * c1), atail, atop);     // (never above the top once the window has been raised: the upper clamp only keeps the address inside the row whatever the data)
            uint32_t u = 1u;
            if (!TOPK) u = (uint32_t)__builtin_amdgcn_exp2f(fmaf(d, c2, fmaf(af, -kLog2ePerBin, ebias)));
            if (key_of(r, hf) < skip) u = 0u;
            lds_add_u32((uint32_t)fmaf(af, -4.0f, abase), u);
          }
        }
      }
    }
  };

  u32x4 pa[LOADS];
  T.fetch(pa, khead, I.tok_stride, tile_origin(c.t_begin + min(wave, n_tiles - 1) * 32, c.t_end), lane);
  for (int tile = wave; tile < n_tiles; tile += kWaves) tile_body(pa, tile);
  if (lane < 32) {
    atomicMax(&S->rowmax[col], ordered_bits(mxrun[0]));
    if (TWO) atomicMax(&S->rowmax[32 + col], ordered_bits(mxrun[1]));
  }
  // this wave is out of tiles; keep serving the others' events until every wave is
  if (lane == 0) atomicAdd(&S->done, 1);
  for (int spins = 0;; ++spins) {
    if (__builtin_amdgcn_readfirstlane(*pending) != 0) {
      sync_event();
    } else if (__builtin_amdgcn_readfirstlane(*done) >= kWaves) {
      break;
    }
    if (spins >= tab.spin_limit) {    // never reached if the protocol holds; a stuck wave must not hang the GPU.
      // Give up VISIBLY: the flag is read by every wave after the workgroup's closing barrier (which this
      // wave now joins; waves still inside an event pair up with it and finish on their own, because ended
      // waves no longer count at a barrier), the workgroup then publishes kTopGaveUp for all its rows and
      // find_bin hands those rows to the exact selector.  Events count as polls, so the loop is bounded.
      if (lane == 0) *(volatile int *)&S->aborted = 1;
      break;
    }
    __builtin_amdgcn_s_sleep(1);
  }
}

template <int DK, bool TOPK, bool NT>
__global__ __launch_bounds__(kThreads) void score_hist_kernel(const FastTable tab) {
  __shared__ __align__(16) unsigned char tiles[kWaves][Tile<DK, true>::BYTES];
  __shared__ uint32_t hist[64 * (kBins + 1)];
  __shared__ HistCtl ctl;
  int wg_id = blockIdx.x;
  if (!xcd_order(tab, wg_id)) return;
  const WgCoord c = decode_wg(tab, wg_id);
  const FastItem I = tab.it[c.it];
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  for (int i = tid; i < 64 * (kBins + 1); i += kThreads) hist[i] = 0u;
  if (tid < 64) {
    ctl.top[tid] = kTopUnset;
    ctl.newmax[tid] = ordered_bits(-3.0e38f);
    ctl.rowmax[tid] = ordered_bits(-3.0e38f);
  }
  if (tid == 0) { ctl.pending = 0; ctl.done = 0; ctl.aborted = 0; }
  if (blockIdx.x == 0 && tid < kRefineLevels + 1) tab.n_refine[tid] = 0;     // (find_bin_kernel counts into it after this kernel)
  __syncthreads();
  if (c.n0 + 32 < tab.NQ)
    hist_fused_body<DK, true, TOPK, NT>(tab, c, I, tiles[wave], hist, &ctl);
  else
    hist_fused_body<DK, false, TOPK, NT>(tab, c, I, tiles[wave], hist, &ctl);
  __syncthreads();
  const int rows = min(64, tab.NQ - c.n0);
  const bool gave_up = *(volatile int *)&ctl.aborted != 0;
  if (tid < rows) {
    tab.part_max[(size_t)c.slot * tab.NQ + c.n0 + tid] = from_ordered_bits(ctl.rowmax[tid]);
    tab.part_top[(size_t)c.slot * tab.NQ + c.n0 + tid] = gave_up ? kTopGaveUp : ctl.top[tid];
  }
  if (gave_up) return;            // (wave-uniform: read after the barrier)
  uint32_t *out = tab.part_hist + ((size_t)c.slot * tab.NQ + c.n0) * kBins;
  for (int i = tid; i < rows * kBins; i += kThreads) out[i] = hist[(i / kBins) * (kBins + 1) + (i % kBins)];
}

// ------------------------------------------------------------------ per row: bin of the cut.  One wave per row.
constexpr int kFindWaves = 4;
// The lanes share out the chunks' maxima and window tops; the histograms are merged GROUP chunks at a time, every load
// of a group issued before any is used, so that their latencies overlap (GROUP = 2 when no item of the call has more
// than two chunks, the large-batch case, where registers cost occupancy; else 4).
template <int GROUP>
__global__ __launch_bounds__(kFindWaves * 64) void find_bin_kernel(const FastTable tab, int n_rows) {
  const int lane = threadIdx.x & 63;
  const int grow = blockIdx.x * kFindWaves + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  if (grow >= n_rows) return;
  const int it = grow / tab.rows_per_item, r = grow - it * tab.rows_per_item;
  const int s = r / tab.Hq, h = r - s * tab.Hq;
  const int kvh = h / tab.G, g = h - kvh * tab.G;
  const int n = s * tab.G + g;
  const FastItem I = tab.it[it];
  const size_t slot0 = (size_t)(I.part0 + kvh * I.n_chunks);
  float m = -INFINITY;
  int top = kTopUnset;
  bool gave_up = false;
  int tc_lane = kTopUnset;            // window top of chunk `lane`
  for (int ch = lane; ch < I.n_chunks; ch += 64) {
    m = fmaxf(m, tab.part_max[(slot0 + ch) * tab.NQ + n]);
    const int tc = tab.part_top[(slot0 + ch) * tab.NQ + n];
    if (ch < 64) tc_lane = tc;
    gave_up = gave_up || tc == kTopGaveUp;
    top = max(top, tc);
  }
  for (int off = 32; off > 0; off >>= 1) {
    m = fmaxf(m, __shfl_xor(m, off, 64));
    top = max(top, __shfl_xor(top, off, 64));
  }
  gave_up = __any(gave_up);
  RowInfo *info = tab.info + grow;
  if (gave_up) {      // a pass-1 workgroup of this row gave up: no histogram to trust, the exact selector redoes the row
    if (lane == 0) {
      info->mdot = m;
      info->astar = 0x7FFFFFFF;   // pass 2 ignores the row
      info->shift = 0;
      info->flag = 7;
      info->above = 0.0;
      info->target = 0.0;
      tab.ovf_cnt[grow] = 0;
    }
  }
  // Every chunk binned inside its own window; on the absolute grid its bin jl is global bin
  // jl + (top - top_chunk).  Weights are fixed-point sums relative to the bin's upper edge, so the
  // chunks' sums of one absolute bin simply add: mass = sum * 2^-kFixBits * exp2(edge - max) in log2
  // units.  Chunk bins at or beyond the last global bin (and the chunks' own last bins) all fall into
  // the last global bin.  A lane owns bins lane, lane + 64, lane + 128, ...
  const bool topk = tab.mode == GVOTE_SELECT_TOPK;
  const double mref = (double)m * (double)tab.c2;
  constexpr int BPL = kBins / 64;     // bins per lane
  unsigned long long acc[BPL];
#pragma unroll
  for (int i = 0; i < BPL; ++i) acc[i] = 0ull;
  float tailpart = 0.f;    // this lane's share of the last global bin, relative to that bin's edge
  // GROUP chunks at a time; the last group repeats its last chunk with weight zero
  for (int ch0 = 0; ch0 < I.n_chunks; ch0 += GROUP) {
    int shift[GROUP];
    const uint32_t *hc[GROUP];
#pragma unroll
    for (int u = 0; u < GROUP; ++u) {
      const int ch = min(ch0 + u, I.n_chunks - 1);
      // (the first 64 chunks' tops are still in the lanes that fetched them: no second, dependent load)
      const int tc = ch < 64 ? __builtin_amdgcn_readlane(tc_lane, ch) : tab.part_top[(slot0 + ch) * tab.NQ + n];
      shift[u] = top - tc;             // >= 0; tops are bounded, the difference fits
      hc[u] = tab.part_hist + ((slot0 + ch) * tab.NQ + n) * kBins;
    }
    uint32_t hu[GROUP][BPL], hv[GROUP][BPL];
#pragma unroll
    for (int u = 0; u < GROUP; ++u) {
#pragma unroll
      for (int i = 0; i < BPL; ++i) {
        const int j = lane + 64 * i;
        hu[u][i] = hc[u][j];                                          // chunk bin j
        hv[u][i] = hc[u][min(max(j - shift[u], 0), kBins - 1)];       // chunk bin that lands in my global bin j (a valid bin whatever the workspace holds)
      }
    }
#pragma unroll
    for (int u = 0; u < GROUP; ++u) {
      const bool live = ch0 + u < I.n_chunks;
#pragma unroll
      for (int i = 0; i < BPL; ++i) {
        const int j = lane + 64 * i;
        const int over = min(j + shift[u] - (kBins - 1), 1 << 20);   // >= 0: it lands in or beyond the last global bin
        const float wt = (float)hu[u][i] * (topk ? 1.0f : __builtin_amdgcn_exp2f(-(float)over * kLog2ePerBin));
        tailpart += (live && over >= 0) ? wt : 0.f;
        acc[i] += (live && j < kBins - 1 && j - shift[u] >= 0) ? hv[u][i] : 0u;
      }
    }
  }
  for (int off = 32; off > 0; off >>= 1) tailpart += __shfl_xor(tailpart, off, 64);
  double mine[BPL];
#pragma unroll
  for (int i = 0; i < BPL; ++i) {
    const int j = lane + 64 * i;
    if (topk) {              // key counts
      mine[i] = j == kBins - 1 ? (double)tailpart : (double)acc[i];
    } else {
      mine[i] = acc[i] ? ldexp((double)acc[i], -kFixBits) * exp2((double)(top - j + 1) * (double)kLog2ePerBin - mref) : 0.0;
      if (j == kBins - 1)
        mine[i] = ldexp((double)tailpart, -kFixBits) * exp2((double)(top - (kBins - 1) + 1) * (double)kLog2ePerBin - mref);
    }
  }
  // inclusive scan over bins (bin 0 = highest logits): within each group of 64 bins, then across groups
  double cum[BPL], base = 0.0;
#pragma unroll
  for (int i = 0; i < BPL; ++i) {
    double x = mine[i];
    for (int off = 1; off < 64; off <<= 1) {
      const double y = __shfl_up(x, off, 64);
      if (lane >= off) x += y;
    }
    cum[i] = base + x;
    base += __shfl(x, 63, 64);
  }
  const double Z = base;
  double target = (double)tab.p * Z;
  if (topk) {
    int k = tab.k_per_row[(size_t)(tab.item0 + it) * tab.rows_per_item + r];
    k = k < 1 ? 1 : (k > I.L ? I.L : k);
    target = (double)k;
  }
  bool found = false;
#pragma unroll
  for (int i = 0; i < BPL; ++i) {
    const int j = lane + 64 * i;
    const double before = cum[i] - mine[i];
    found = found || (before < target && cum[i] >= target);
    if (!gave_up && before < target && cum[i] >= target) {
      info->mdot = m;
      info->astar = top - j;
      info->shift = 0;
      int flag = (j == kBins - 1) ? 1 : 0;      // 1: the cut lies below the histogram window
      // keys in the cut bin: every key adds between 0.94 and 1 times 2^kFixBits to its bin (weights are relative to
      // the bin's own upper edge), so the fixed-point sum also counts them.  More than the resolver can hold
      // (flat attention over a long context): look inside the bin with 256 finer bins first.
      // Pass 2 collects the bin's keys in n_sub = I.n_chunks * emit_split * 2 * kWaves private lists of kSubCap = 16
      // entries per row plus kOvfCap = 256 shared ones.  With an average fill f the lists spill about
      // n_sub * E[(Poisson(f) - 16)+] entries: 3.0 per list at f = 18, 1.0 at 15, 0.3 at 13, 0.06 at 11 - the fills
      // below keep the spill under 200.  (A second pass over K for a block costs less than one row in the exact
      // selector, but far more than a bin that fits.)
      const double in_bin = (topk ? mine[i] : (double)acc[i] * (1.0 / (double)(1 << kFixBits))) * 1.07;
      const int n_sub = I.n_chunks * tab.emit_split * 2 * kWaves;
      const double fill = n_sub <= 64 ? 18.0 : (n_sub <= 160 ? 15.0 : (n_sub <= 512 ? 13.0 : 11.0));
      const double room = fmin((double)kFineTrigger, fill * (double)n_sub);
      if (flag == 0 && in_bin > room && abs(top - j) < kFineSpan) flag = 4;    // (beyond kFineSpan the row goes on as it is)
      info->flag = flag;
      if (flag != 0) atomicAdd(tab.n_refine, 1);     // asks for a second histogram (score_refine_kernel)
      info->above = before;
      info->target = target;
    }
  }
  if (!gave_up && !__any(found)) {      // cannot happen (Z holds at least the largest key's weight, a count is at least 1): never
    if (lane == 0) {                    // leave a row without a record, hand it to the exact selector like a row that gave up
      info->mdot = m;
      info->astar = 0x7FFFFFFF;
      info->shift = 0;
      info->flag = 7;
      info->above = 0.0;
      info->target = 0.0;
    }
  }
  if (lane == 0) {
    tab.ovf_cnt[grow] = 0;
    if (grow == 0) {
      if (tab.item0 == 0) {
        *tab.n_fallback = 0;
        tab.n_list[1] = 0; tab.n_list[2] = 0; tab.n_list[3] = 0; tab.n_list[4] = 0; tab.n_list[5] = 0;
      }
      *tab.n_list = 0;
    }
    const size_t gr = (size_t)(tab.item0 + it) * tab.rows_per_item + r;
    if (tab.row_max) tab.row_max[gr] = m * tab.scale;
    if (tab.row_sum) tab.row_sum[gr] = (float)Z;
  }
}

// ------------------------------------------------------------------ deeper windows for rows whose cut lies below the first
// A row whose cut falls into the last bin of its 256-bin window (flag 1: a far-reaching p, or one dominant key
// over a long flat tail) gets another window right below the first: the same absolute grid, the window top
// fixed at the first window's last bin (so nothing slides and no wave waits for another), keys above it
// ignored - their weight is already in `above`.  Only workgroups with such a row in their block of 64 do
// anything.  refine_bin_kernel then continues the row's cumulative search in the new bins; a row that is
// still in a last bin keeps flag 1 and can be refined again.
template <int DK, bool TWO, bool TOPK, bool NT>
__device__ __forceinline__ void hist_fixed_body(const FastTable &tab, const WgCoord &c, const FastItem &I,
                                                unsigned char *ldstile, uint32_t *hist, const int *top_s, const int *shift_s) {
  constexpr int LOADS = Tile<DK, true>::LOADS;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hf = lane >> 5,
            col = lane & 31;
  Tile<DK, NT> T;
  T.load_q(tab, c.it, c.kvh, c.n0, lane);
  const bf16_t *khead = reinterpret_cast<const bf16_t *>(I.k) + (long long)c.kvh * I.head_stride;
  const int n_tiles = (c.t_end - c.t_begin + 31) >> 5;
  const int last_tile = wave < n_tiles ? wave + kWaves * ((n_tiles - 1 - wave) / kWaves) : n_tiles - 1;
  const float c2 = tab.c2;
  uint32_t *hrow[2] = {hist + col * (kBins + 1), hist + (32 + col) * (kBins + 1)};
  // rows that are not being refined keep a harmless window (top 0) and a ceiling no key passes
  const int top[2] = {top_s[col], top_s[32 + col]};
  // a row's bins are 2^-shift standard bins wide (scaling by a power of two is exact: floor(d c1 2^shift) is the
  // same number pass 2 compares against)
  const float c1r[2] = {ldexpf(tab.c1, shift_s[col]), ldexpf(tab.c1, shift_s[32 + col])};
  const float kr[2] = {ldexpf(kLog2ePerBin, -shift_s[col]), ldexpf(kLog2ePerBin, -shift_s[32 + col])};
  const bool live[2] = {top[0] != kTopUnset, top[1] != kTopUnset};
  u32x4 pre[LOADS];
  T.fetch(pre, khead, I.tok_stride, tile_origin(c.t_begin + min(wave, n_tiles - 1) * 32, c.t_end), lane);
  for (int tile = wave; tile < n_tiles; tile += kWaves) {
    const int t0 = c.t_begin + tile * 32;
    const int skip = t0 - tile_origin(t0, c.t_end);
    floatx16 acc[2];
    T.stage(pre, ldstile, lane);
    {
      const int tn = c.t_begin + min(tile + kWaves, last_tile) * 32;
      T.fetch(pre, khead, I.tok_stride, tile_origin(tn, c.t_end), lane);
    }
    __builtin_amdgcn_wave_barrier();
    T.template compute<TWO>(acc, ldstile, lane);
    __builtin_amdgcn_wave_barrier();
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      if (nb == 0 || TWO) {
        const int tp = live[nb] ? top[nb] : 0;
        const float atop = (float)tp, atail = (float)(tp - (kBins - 1));
        const float ceil_f = live[nb] ? atop : -INFINITY;       // keys in bins above this are not counted here
        const float abase = (float)(lds_offset(hrow[nb]) + 4 * tp);
        const float c1 = c1r[nb], nk = -kr[nb], ebias = (float)kFixBits - kr[nb];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float d = acc[nb][r];
          const float a = floorf(d * c1);
          const float af = fminf(fmaxf(a, atail), atop);
          uint32_t u = 1u;
          if (!TOPK) u = (uint32_t)__builtin_amdgcn_exp2f(fmaf(d, c2, fmaf(af, nk, ebias)));
          if (!(a <= ceil_f) || key_of(r, hf) < skip) u = 0u;
          lds_add_u32((uint32_t)fmaf(af, -4.0f, abase), u);
          if ((r & 3) == 3) __builtin_amdgcn_sched_barrier(0);
        }
      }
    }
  }
}

template <int DK, bool TOPK, bool NT>
__global__ __launch_bounds__(kThreads) void score_refine_kernel(const FastTable tab, int level) {
  __shared__ __align__(16) unsigned char tiles[kWaves][Tile<DK, true>::BYTES];
  __shared__ uint32_t hist[64 * (kBins + 1)];
  __shared__ int top_s[64], shift_s[64];
  __shared__ int any_s;
  if (tab.n_refine[level] == 0) return;    // nobody asked (the usual case): one scalar load per workgroup
  int wg_id = blockIdx.x;
  if (!xcd_order(tab, wg_id)) return;
  const WgCoord c = decode_wg(tab, wg_id);
  const FastItem I = tab.it[c.it];
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  if (tid == 0) any_s = 0;
  __syncthreads();
  if (tid < 64) {
    int t = kTopUnset, sh = 0;
    const int n = c.n0 + tid;
    if (n < tab.NQ) {
      const int s = n / tab.G, g = n % tab.G;
      const RowInfo &ri = tab.info[c.it * tab.rows_per_item + s * tab.Hq + c.kvh * tab.G + g];
      // (bin numbers stay far inside +-2^21, where 4 * top + LDS offset is exact in fp32; anything else is not a
      // record find_bin wrote and is left alone)
      if (ri.flag == 1 && abs(ri.astar) < (1 << 21)) { t = ri.astar; any_s = 1; }      // astar of a flag-1 row = its window's last bin
      if (ri.flag == 4 && abs(ri.astar) < kFineSpan) { t = (ri.astar + 1) * kFineBins - 1; sh = kFineShift; any_s = 1; }   // the finest bin under the cut bin's upper edge
    }
    top_s[tid] = t;
    shift_s[tid] = sh;
  }
  for (int i = tid; i < 64 * (kBins + 1); i += kThreads) hist[i] = 0u;
  __syncthreads();
  if (any_s == 0) return;                  // (uniform: read after the barrier)
  if (c.n0 + 32 < tab.NQ)
    hist_fixed_body<DK, true, TOPK, NT>(tab, c, I, tiles[wave], hist, top_s, shift_s);
  else
    hist_fixed_body<DK, false, TOPK, NT>(tab, c, I, tiles[wave], hist, top_s, shift_s);
  __syncthreads();
  const int rows = min(64, tab.NQ - c.n0);
  uint32_t *out = tab.part_hist + ((size_t)c.slot * tab.NQ + c.n0) * kBins;
  for (int i = tid; i < rows * kBins; i += kThreads) out[i] = hist[(i / kBins) * (kBins + 1) + (i % kBins)];
}

// one wave per row: continue the cumulative search of a flagged row in its second histogram
__device__ __forceinline__ void refine_row(const FastTable &tab, int grow, int level, int lane) {
  RowInfo *info = tab.info + grow;
  if (info->flag != 1 && info->flag != 4) return;
  if ((info->flag == 1 && abs(info->astar) >= (1 << 21)) || (info->flag == 4 && abs(info->astar) >= kFineSpan)) {
    if (lane == 0 && info->flag == 4) info->flag = 5;    // (score_refine_kernel left such a record alone: the exact selector takes the row)
    return;
  }
  const int it = grow / tab.rows_per_item, r = grow - it * tab.rows_per_item;
  const int s = r / tab.Hq, h = r - s * tab.Hq;
  const int kvh = h / tab.G, g = h - kvh * tab.G;
  const int n = s * tab.G + g;
  const FastItem I = tab.it[it];
  const size_t slot0 = (size_t)(I.part0 + kvh * I.n_chunks);
  const bool topk = tab.mode == GVOTE_SELECT_TOPK;
  const bool fine = info->flag == 4;
  const int sh = fine ? kFineShift : 0;
  const int top = fine ? (info->astar + 1) * kFineBins - 1 : info->astar;
  const double kr = ldexp((double)kLog2ePerBin, -sh);
  const double mref = (double)info->mdot * (double)tab.c2;
  constexpr int BPL = kBins / 64;
  double mine[BPL];
#pragma unroll
  for (int i = 0; i < BPL; ++i) {
    const int j = lane + 64 * i;
    unsigned long long a = 0ull;
    for (int ch = 0; ch < I.n_chunks; ++ch) a += tab.part_hist[((slot0 + ch) * tab.NQ + n) * kBins + j];
    mine[i] = topk ? (double)a
                   : (a ? ldexp((double)a, -kFixBits) * exp2((double)(top - j + 1) * kr - mref) : 0.0);
  }
  double cum[BPL], base = info->above;
#pragma unroll
  for (int i = 0; i < BPL; ++i) {
    double x = mine[i];
    for (int off = 1; off < 64; off <<= 1) {
      const double y = __shfl_up(x, off, 64);
      if (lane >= off) x += y;
    }
    cum[i] = base + x;
    base += __shfl(x, 63, 64);
  }
  const double target = info->target;
  // (fixed-point truncation can leave the refined bins a hair short of the first window's last bin: a target
  // that no bin reaches stays with the last bin)
  const bool reached = base >= target;
  __builtin_amdgcn_wave_barrier();
#pragma unroll
  for (int i = 0; i < BPL; ++i) {
    const int j = lane + 64 * i;
    const double before = cum[i] - mine[i];
    const bool here = reached ? (before < target && cum[i] >= target) : (j == kBins - 1);
    if (here) {
      info->astar = top - j;
      info->shift = sh;
      info->above = before;
      // (inside a cut bin the last fine bin also collects every key below the bin, which cannot matter: the bin as a
      // whole reaches the target, so a crossing found there is the true one and `before` is exact)
      if (j != kBins - 1 || fine) {
        info->flag = 0;
        atomicAdd(tab.n_list + 5, 1);                 // diagnostic: rows settled by a deeper window
      } else {
        atomicAdd(tab.n_refine + level + 1, 1);       // still below: next level, or the exact selector
      }
    }
  }
}

// a small grid walks the rows (the launch costs little when nobody asked)
constexpr int kRefineBinGrid = 512;
__global__ __launch_bounds__(kFindWaves * 64) void refine_bin_kernel(const FastTable tab, int n_rows, int level) {
  if (tab.n_refine[level] == 0) return;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  for (int grow = blockIdx.x * kFindWaves + wave; grow < n_rows; grow += gridDim.x * kFindWaves) refine_row(tab, grow, level, lane);
}

// ------------------------------------------------------------------ pass 2: masks + boundary candidates
// Pass 1 left the maximum of every (tile, row).  A tile in which no row reaches its cut bin selects
// nothing, so its keys are not even fetched: the second K read shrinks to the tiles that matter
// (attention mass is concentrated, most tiles hold no selected key for any of the 64 rows).
constexpr int kMaxChunkWords = 8 * kRoundKeys / 32;     // mask words per row of the largest pass-2 piece (256)
struct EmitShared {
  uint32_t mwords[64][kMaxChunkWords + 1];
  int astar[64];    // the cut bin on the standard grid (the tile test), 0x7FFFFFFF for rows pass 2 leaves alone
  float lo[64], hi[64];   // d * c1 in [lo, hi): the key lies in the row's cut bin; >= hi: above it (the bin may be a fine one)
  int row[64];      // row index (s * H_q + h) of the workgroup's 64 query rows, -1 if absent
  int n_need, next;                       // tiles of the piece that pass 2 has to look at, and how many have been taken
  uint32_t need_w[kWaves];                // per wave: which of its tiles
  unsigned short tlist[kMaxChunkWords];   // ... their numbers inside the piece
};

template <int DK, bool TWO, bool NT>
__device__ __forceinline__ void emit_body(const FastTable &tab, const WgCoord &c, const FastItem &I,
                                          unsigned char *ldstile, EmitShared *E) {
  constexpr int LOADS = Tile<DK, true>::LOADS;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6), hf = lane >> 5,
            col = lane & 31;
  const int row_base = c.it * tab.rows_per_item;
  Tile<DK, NT> T;
  T.load_q(tab, c.it, c.kvh, c.n0, lane);
  const bf16_t *khead = reinterpret_cast<const bf16_t *>(I.k) + (long long)c.kvh * I.head_stride;
  const float c1 = tab.c1;
  const float lo_r[2] = {E->lo[col], E->lo[32 + col]}, hi_r[2] = {E->hi[col], E->hi[32 + col]};
  const int grow[2] = {row_base + E->row[col], row_base + E->row[32 + col]};   // only used for rows that exist
  const int n_tiles = (c.t_end - c.t_begin + 31) >> 5;
  const int nk = wave < n_tiles ? (n_tiles - wave + kWaves - 1) / kWaves : 0;   // tiles of this wave (<= 32)

  // which of my tiles hold a key in or above some row's cut bin?  (a = floor(d c1) is monotone in d, so the
  // bin of a tile's largest dot says it exactly)
  uint32_t need = 0u;
  {
    const int a_l = E->astar[lane];      // 0x7FFFFFFF for absent rows and rows the exact selector redoes
    const short *tm = tab.tile_bin + I.tmax0 + ((size_t)c.kvh * I.W + (c.t_begin >> 5)) * tab.NQ + c.n0 + lane;
    const bool row_ok = c.n0 + lane < tab.NQ;
    // all loads first (independent, in flight together), then the votes
    constexpr int kMaxK = 32;          // chunk_keys <= 8192 -> at most 32 tiles per wave
    int v[kMaxK];
#pragma unroll
    for (int k = 0; k < kMaxK; ++k)
      v[k] = (row_ok && k < nk) ? (int)tm[(size_t)(wave + kWaves * k) * tab.NQ] : -32768;
#pragma unroll
    for (int k = 0; k < kMaxK; ++k)
      if (__any(v[k] >= a_l)) need |= 1u << k;
  }

  // Candidate sub-lists: one per (row, key chunk, wave, lane half), written by exactly one lane, so the
  // count lives in a register and nothing waits on an atomic's return.
  const int sub = (c.chunk * kWaves + wave) * 2 + hf;
  int ccount[2] = {0, 0};
  uint2 *cdst[2];
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) cdst[nb] = tab.cands + ((size_t)grow[nb] * tab.sub_per_row + sub) * kSubCap;

  // The tiles to look at go into one list for the workgroup; the waves then take them one at a time from a
  // shared counter, so a wave whose own tiles mostly drop out helps with the others' (the tiles that matter
  // are clustered).  No workgroup barrier inside the loop.
  // The list is in ascending key order (the same on every run; the row blocks of one chunk, which run side by side,
  // sweep the keys together).
  if (lane == 0) E->need_w[wave] = need;
  __syncthreads();
  {
    // tile wave + 8 k comes after every tile (w', k') with k' < k, and after those with k' == k and w' < wave
    int before = 0, total = 0;
    const uint32_t lower = lane < 32 ? (1u << lane) - 1u : 0xFFFFFFFFu;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      const uint32_t nw = E->need_w[w];
      total += __popc(nw);
      before += __popc(nw & lower) + ((w < wave && lane < 32) ? (int)((nw >> lane) & 1u) : 0);
    }
    if (lane < 32 && ((need >> lane) & 1u)) E->tlist[before] = (unsigned short)(wave + kWaves * lane);
    if (threadIdx.x == 0) E->n_need = total;
  }
  __syncthreads();
  const int n_need = E->n_need;
  volatile lds_int *next = (volatile lds_int *)(size_t)lds_offset(&E->next);
  auto next_k = [&]() __attribute__((always_inline)) -> int {
    int gi = 0;
    if (lane == 0) gi = __hip_atomic_fetch_add((lds_int *)next, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    gi = __builtin_amdgcn_readfirstlane(gi);
    return gi < n_need ? (int)E->tlist[gi] : -1;
  };
  auto process = [&](u32x4(&pre)[LOADS], int tile, int tile_refill) __attribute__((always_inline)) {
    const int t0 = c.t_begin + tile * 32;
    const int org = tile_origin(t0, c.t_end);
    const int skip = t0 - org;          // leading keys of the loaded window that are not this tile's
    T.stage(pre, ldstile, lane);
    {   // refill with the next tile to look at (or this one again: no conditional load)
      const int tn = c.t_begin + (tile_refill >= 0 ? tile_refill : tile) * 32;
      T.fetch(pre, khead, I.tok_stride, tile_origin(tn, c.t_end), lane);
    }
    __builtin_amdgcn_wave_barrier();
    floatx16 acc[2];
    T.template compute<TWO>(acc, ldstile, lane);
    __builtin_amdgcn_wave_barrier();
    // floor(d * c1) >= astar  <=>  d * c1 >= astar (astar is an integer): two compares, no floor
    uint32_t ge[2] = {0u, 0u}, gt[2] = {0u, 0u};
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      if (nb == 0 || TWO) {
        const float lo = lo_r[nb], hi = hi_r[nb];
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const float x = acc[nb][r] * c1;
          ge[nb] |= x >= lo ? (1u << key_of(r, hf)) : 0u;
          gt[nb] |= x >= hi ? (1u << key_of(r, hf)) : 0u;
        }
      }
    }
    if (skip) {                          // wave-uniform: a pulled-back last tile
      const uint32_t mine = 0xFFFFFFFFu << skip;
      ge[0] &= mine; ge[1] &= mine; gt[0] &= mine; gt[1] &= mine;
    }
    const uint32_t cm[2] = {ge[0] & ~gt[0], ge[1] & ~gt[1]};
    if (__any((cm[0] | cm[1]) != 0u)) {   // keys inside a cut bin go to this lane's own sub-lists: no atomics
      // accumulator registers 4g .. 4g+3 hold four neighbouring keys: one wave-uniform test per group
#pragma unroll
      for (int nb = 0; nb < 2; ++nb) {
#pragma unroll
        for (int g = 0; g < 4; ++g) {
          const uint32_t grp = (cm[nb] >> (8 * g + 4 * hf)) & 0xFu;
          if (__any(grp != 0u)) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
              if (grp & (1u << i)) {
                const uint2 e = make_uint2(__float_as_uint(acc[nb][4 * g + i]), (uint32_t)(org + 8 * g + 4 * hf + i));
                if (ccount[nb] < kSubCap) {
                  cdst[nb][ccount[nb]] = e;
                } else {                       // rare: this lane's sub-list is full, use the row's shared list
                  const int slot = atomicAdd(&tab.ovf_cnt[grow[nb]], 1);
                  if (slot < kOvfCap) tab.ovf[(size_t)grow[nb] * kOvfCap + slot] = e;
                  else tab.info[grow[nb]].flag = 3;   // 3: even the overflow list is full, the exact selector redoes the row
                }
                ++ccount[nb];
              }
            }
          }
        }
      }
    }
#pragma unroll
    for (int nb = 0; nb < 2; ++nb) {
      const uint32_t w = (gt[nb] | __shfl_xor(gt[nb], 32, 64)) >> skip;   // bit i = key t0 + i
      if (lane < 32 && w != 0u) E->mwords[32 * nb + lane][tile] = w;
    }
  };

  u32x4 pa[LOADS], pb[LOADS];
  int ka = next_k(), kb = next_k();
  if (ka >= 0) {
    T.fetch(pa, khead, I.tok_stride, tile_origin(c.t_begin + ka * 32, c.t_end), lane);
    T.fetch(pb, khead, I.tok_stride, tile_origin(c.t_begin + (kb >= 0 ? kb : ka) * 32, c.t_end), lane);
  }
  while (ka >= 0) {
    const int ka2 = next_k();
    process(pa, ka, ka2);
    if (kb >= 0) {
      const int kb2 = next_k();
      process(pb, kb, kb2);
      kb = kb2;
    }
    ka = ka2;
  }
#pragma unroll
  for (int nb = 0; nb < 2; ++nb) {
    if ((nb == 0 || TWO) && c.n0 + 32 * nb + col < tab.NQ) {
      tab.cand_cnt[(size_t)grow[nb] * tab.sub_per_row + sub] = min(ccount[nb], kSubCap);
    }
  }
  __syncthreads();
  // the chunk's mask words: every row writes one contiguous run (up to 1 KiB)
  const int w_first = c.t_begin >> 5;
  for (int nl = tid >> 3; nl < 64; nl += kThreads >> 3) {      // eight threads per row, 32-byte runs
    const int r = E->row[nl];
    if (r >= 0) {
      uint32_t *dst = tab.rowmask + I.mask_off + (long long)r * I.W + w_first;
      for (int w = tid & 7; w < n_tiles; w += 8) dst[w] = E->mwords[nl][w];
    }
  }
}

template <int DK, bool NT>
__global__ __launch_bounds__(kThreads) void score_emit_kernel(const FastTable tab) {
  __shared__ __align__(16) unsigned char tiles[kWaves][Tile<DK, true>::BYTES];
  __shared__ EmitShared E;
  int wg_id = blockIdx.x / tab.emit_split;
  const int piece = blockIdx.x - wg_id * tab.emit_split;
  if (!xcd_order(tab, wg_id)) return;
  WgCoord c = decode_wg(tab, wg_id);
  const FastItem I = tab.it[c.it];
  {   // this workgroup's piece of the chunk (possibly empty at the end of an item: its counts are still written)
    const int piece_keys = tab.chunk_keys / tab.emit_split;
    c.t_begin = min(c.t_begin + piece * piece_keys, c.t_end);
    c.t_end = min(c.t_end, c.t_begin + piece_keys);
    c.chunk = c.chunk * tab.emit_split + piece;     // numbers the candidate sub-lists
  }
  const int tid = threadIdx.x, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int row_base = c.it * tab.rows_per_item;   // batch-local row index of (s = 0, h = 0)
  if (tid < 64) {
    const int n = c.n0 + tid;
    int a = 0x7FFFFFFF, r = -1;
    float lo = 3.0e38f, hi = 3.0e38f;
    if (n < tab.NQ) {
      const int s = n / tab.G, g = n % tab.G;
      r = s * tab.Hq + c.kvh * tab.G + g;
      const RowInfo &ri = tab.info[row_base + r];
      a = ri.astar;
      if (a != 0x7FFFFFFF) {
        lo = ldexpf((float)a, -ri.shift);            // exact: |a| < 2^24
        hi = ldexpf((float)a + 1.0f, -ri.shift);
        a >>= ri.shift;                               // (arithmetic shift = floor: the standard bin that holds the fine one)
        a = min(a, 32767);                            // pass 1 stored the tile bins as int16, saturated: a saturated tile must pass the test
      }
    }
    if (tid == 0) { E.n_need = 0; E.next = 0; }
    E.astar[tid] = a;
    E.lo[tid] = lo;
    E.hi[tid] = hi;
    E.row[tid] = r;
  }
  for (int i = tid; i < 64 * (kMaxChunkWords + 1); i += kThreads) (&E.mwords[0][0])[i] = 0u;
  __syncthreads();
  if (c.n0 + 32 < tab.NQ)
    emit_body<DK, true, NT>(tab, c, I, tiles[wave], &E);
  else
    emit_body<DK, false, NT>(tab, c, I, tiles[wave], &E);
}

// ------------------------------------------------------------------ per row: exact cut among the candidates
// One WAVE per row, no workgroup barrier: the row's candidates (the keys inside its cut bin, typically a
// few dozen) are gathered from the sub-lists into wave-private LDS, then an 8-digit radix search over the
// 64-bit key (ordered raw dot, ~position) finds the last key the target needs; weights are fixed point
// relative to the cut bin's edge (integer LDS atomics).
// Rows with at most 64 candidates (the usual case) need no search at all: with one candidate per lane,
// 64 exchange steps give every lane the total weight of the keys ahead of its own; a key is needed iff
// that weight still falls short of the target.  Launched twice: CAP = 256 for everybody (four rows per
// workgroup), then CAP = kCandCap for the rows the first launch marked as larger (flag 2; one row per
// workgroup); rows beyond kCandCap get flag 1.
template <int CAP>
struct ResolveLds {
  unsigned long long key[CAP];
  uint32_t wgt[CAP];
  uint32_t hist[256];
  int hcnt[256];
};

template <int CAP, bool SECOND>
__global__ __launch_bounds__((SECOND ? 1 : 4) * 64) void resolve_kernel(const FastTable tab, int n_rows) {
  constexpr int kResolveWaves = SECOND ? 1 : 4;     // the large second tier needs the LDS of a whole workgroup
  __shared__ ResolveLds<CAP> lds[kResolveWaves];
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int grow = blockIdx.x * kResolveWaves + wave;
  if (grow >= n_rows) return;
  RowInfo *info = tab.info + grow;
  if (SECOND) {                          // the second tier has nothing to do for nearly every row: look before fetching
    const int f = info->flag;
    if (!(f & 1) && f != 2) return;
  }
  // Everything that does not depend on the row's record is requested before the record is looked at: the record
  // itself in one piece, the length of the overflow list and the lengths of the first 256 sub-lists.
  const int it = grow / tab.rows_per_item, r = grow - it * tab.rows_per_item;
  const FastItem I = tab.it[it];
  const int n_sub = I.n_chunks * tab.emit_split * 2 * kWaves;
  const int *ccnt = tab.cand_cnt + (size_t)grow * tab.sub_per_row;
  const uint2 *clist = tab.cands + (size_t)grow * tab.sub_per_row * kSubCap;
  int nn[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) nn[u] = 64 * u + lane < n_sub ? ccnt[64 * u + lane] : 0;
  const int ovf_raw = tab.ovf_cnt[grow];
  const RowInfo R = *info;
  const int flag = R.flag;
  if (SECOND && (flag & 1)) {           // settled as "needs the exact selector": queue the row
    if (lane == 0) {
      tab.row_list[atomicAdd(tab.n_list, 1)] = grow;
      atomicAdd(tab.n_list + 1 + (flag >> 1), 1);      // diagnostic: rows by reason (window, sub-list, capacity, gave up)
    }
    return;
  }
  if (SECOND ? flag != 2 : flag != 0) return;
  ResolveLds<CAP> &M = lds[wave];
  // fixed-point scale: weights relative to the upper edge of the cut bin, 2^kFixBits each at most
  const double edge = ldexp((double)(R.astar + 1) * (double)kLog2ePerBin, -R.shift);       // log2 units
  const float efix = (float)((double)kFixBits - edge);
  const bool topk = tab.mode == GVOTE_SELECT_TOPK;
  const double unit = topk ? 1.0 : exp2((double)R.mdot * (double)tab.c2 - edge) * (double)(1 << kFixBits);
  const double target = R.target * unit;
  double above = R.above * unit;
  auto put = [&](int dst, uint2 e) __attribute__((always_inline)) {
    const float d = __uint_as_float(e.x);
    M.key[dst] = ((unsigned long long)ordered_bits(d) << 32) | (unsigned long long)(0xFFFFFFFFu - e.y);
    M.wgt[dst] = topk ? 1u : (uint32_t)__builtin_amdgcn_exp2f(fmaf(d, tab.c2, efix));
  };
  // the row's shared overflow list: its first 64 entries are on their way while the sub-lists are gathered
  const int n_ovf = max(0, min(ovf_raw, kOvfCap));
  const uint2 ovf_first = lane < n_ovf ? tab.ovf[(size_t)grow * kOvfCap + lane] : make_uint2(0u, 0u);

  // gather the sub-lists (order is irrelevant: keys are unique), 256 of them at a time: their counts are fetched
  // together (those of the next 256 while these are worked on), then the first entry of each (most hold none or
  // one), so that a row does not pay a memory round trip per step
  int cnt = 0;
  for (int s0 = 0; s0 < n_sub; s0 += 256) {
    uint2 first[4];
#pragma unroll
    for (int u = 0; u < 4; ++u)
      first[u] = nn[u] > 0 ? clist[(size_t)(s0 + 64 * u + lane) * kSubCap] : make_uint2(0u, 0u);
    int nn_next[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) nn_next[u] = s0 + 256 + 64 * u + lane < n_sub ? ccnt[s0 + 256 + 64 * u + lane] : 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      if (s0 + 64 * u >= n_sub) break;
      const int n = nn[u];
      int x = n;
      for (int off = 1; off < 64; off <<= 1) {
        const int y = __shfl_up(x, off, 64);
        if (lane >= off) x += y;
      }
      const int dst0 = cnt + x - n;
      const uint2 *src = clist + (size_t)(s0 + 64 * u + lane) * kSubCap;
      for (int i = 0; i < n; ++i)
        if (dst0 + i < CAP) put(dst0 + i, i == 0 ? first[u] : src[i]);
      cnt += __shfl(x, 63, 64);
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) nn[u] = nn_next[u];
  }
  for (int i = lane; i < n_ovf; i += 64)
    if (cnt + i < CAP) put(cnt + i, i < 64 ? ovf_first : tab.ovf[(size_t)grow * kOvfCap + i]);
  cnt += n_ovf;
  if (cnt > CAP) {
    if (lane == 0) {
      info->flag = (!SECOND && cnt <= kCandCap) ? 2 : 5;   // 5: more candidates than the resolver holds
      if (SECOND) {
        tab.row_list[atomicAdd(tab.n_list, 1)] = grow;
        atomicAdd(tab.n_list + 3, 1);
      }
    }
    return;
  }
  if (SECOND && lane == 0) info->flag = 0;
  __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
  uint32_t *mrow = tab.rowmask + I.mask_off + (long long)r * I.W;
  if (cnt <= 64) {
    const bool have = lane < cnt;
    const unsigned long long mykey = have ? M.key[lane] : 0ull;
    const uint32_t myw = have ? M.wgt[lane] : 0u;
    unsigned long long ahead = 0ull;       // fixed-point weight of the candidates ranked before mine
    const uint32_t klo = (uint32_t)mykey, khi = (uint32_t)(mykey >> 32);
    const int n = __builtin_amdgcn_readfirstlane(cnt);
    for (int j = 0; j < n; ++j) {          // j is wave-uniform: lane reads through scalar registers, no LDS traffic
      const unsigned long long kj = ((unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)khi, j) << 32) |
                                    (unsigned long long)(uint32_t)__builtin_amdgcn_readlane((int)klo, j);
      const uint32_t wj = (uint32_t)__builtin_amdgcn_readlane((int)myw, j);
      if (kj > mykey) ahead += wj;
    }
    if (have && above + (double)ahead < target) {
      const uint32_t t = 0xFFFFFFFFu - (uint32_t)(mykey & 0xFFFFFFFFull);
      if (t < (uint32_t)I.L) atomicOr(&mrow[t >> 5], 1u << (t & 31));
    }
    return;
  }
  // The candidates share a bin, hence the leading bytes of their keys: the search starts at the first byte in which
  // two of them differ, and ends as soon as the digit it picks holds a single key (that key is the last one needed).
  unsigned long long diff = 0ull;
  {
    const unsigned long long k0 = M.key[0];
    for (int i = lane; i < cnt; i += 64) diff |= M.key[i] ^ k0;
    for (int off = 32; off > 0; off >>= 1) diff |= __shfl_xor(diff, off, 64);
  }
  const int first_pass = diff ? __clzll((long long)diff) >> 3 : 7;
  unsigned long long prefix = first_pass ? M.key[0] >> (64 - 8 * first_pass) : 0ull;
  for (int pass = first_pass; pass < 8; ++pass) {
    const int shift = 56 - 8 * pass;
#pragma unroll
    for (int i = 0; i < 4; ++i) { M.hist[lane * 4 + i] = 0u; M.hcnt[lane * 4 + i] = 0; }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    for (int i = lane; i < cnt; i += 64) {
      const unsigned long long k = M.key[i];
      if (pass == 0 || (k >> (shift + 8)) == prefix) {
        const int dg = (int)((k >> shift) & 255ull);
        atomicAdd(&M.hist[dg], M.wgt[i]);
        atomicAdd(&M.hcnt[dg], 1);
      }
    }
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    const int pick = pick_digit_wave(M.hist, M.hcnt, above, target, lane);
    prefix = (prefix << 8) | (unsigned long long)(pick & 255);
    const bool single = M.hcnt[pick & 255] == 1;
    __builtin_amdgcn_fence(__ATOMIC_SEQ_CST, "wavefront");
    if (single) {
      prefix <<= shift;      // (the remaining bytes as zeros: the one key of the digit is not below that)
      break;
    }
  }
  for (int i = lane; i < cnt; i += 64) {
    if (M.key[i] >= prefix) {
      const uint32_t t = 0xFFFFFFFFu - (uint32_t)(M.key[i] & 0xFFFFFFFFull);
      if (t < (uint32_t)I.L) atomicOr(&mrow[t >> 5], 1u << (t & 31));
    }
  }
}

constexpr int kMaxChunkKeys = 16 * kRoundKeys;     // pass 1: the 32-bit fixed-point bins hold 16384 keys
constexpr int kMaxEmitKeys = 8 * kRoundKeys;       // pass 2: its LDS mask buffer holds 8192 keys per row
int pick_chunk_keys(const gvote_shape *sh, const gvote_item *items, int n_items) {
  // about two pass-1 workgroups per CU over the batch (per-chunk set-up and the flush of the histograms
  // are not free); a chunk is a whole number of 1024-key rounds
  long long keys = 0;
  for (int i = 0; i < n_items; ++i) keys += (long long)items[i].L * sh->n_kv_heads;
  long long ck = (keys + 511) / 512;
  ck = (ck + kRoundKeys - 1) / kRoundKeys * kRoundKeys;
  if (ck < kRoundKeys) ck = kRoundKeys;
  if (ck > kMaxChunkKeys) ck = kMaxChunkKeys;
  return (int)ck;
}
// pass 1, the cut bins, the second histogram for the rows that asked, pass 2
template <int DK, bool NT>
gvote_status launch_passes(const FastTable &tab, int grid_wg, int rows, bool topk, hipStream_t st) {
  if (topk) hipLaunchKernelGGL((score_hist_kernel<DK, true, NT>), dim3(grid_wg), dim3(kThreads), 0, st, tab);
  else hipLaunchKernelGGL((score_hist_kernel<DK, false, NT>), dim3(grid_wg), dim3(kThreads), 0, st, tab);
  GVOTE_CHECK_LAUNCH();
  if (tab.sub_per_row > 2 * tab.emit_split * 2 * kWaves)      // (= the call's largest chunk count is above two)
    hipLaunchKernelGGL(find_bin_kernel<4>, dim3(ceil_div(rows, kFindWaves)), dim3(kFindWaves * 64), 0, st, tab, rows);
  else
    hipLaunchKernelGGL(find_bin_kernel<2>, dim3(ceil_div(rows, kFindWaves)), dim3(kFindWaves * 64), 0, st, tab, rows);
  GVOTE_CHECK_LAUNCH();
  for (int lvl = 0; lvl < kRefineLevels; ++lvl) {
    if (topk) hipLaunchKernelGGL((score_refine_kernel<DK, true, NT>), dim3(grid_wg), dim3(kThreads), 0, st, tab, lvl);
    else hipLaunchKernelGGL((score_refine_kernel<DK, false, NT>), dim3(grid_wg), dim3(kThreads), 0, st, tab, lvl);
    GVOTE_CHECK_LAUNCH();
    hipLaunchKernelGGL(refine_bin_kernel, dim3(min(ceil_div(rows, kFindWaves), kRefineBinGrid)), dim3(kFindWaves * 64), 0, st, tab,
                       rows, lvl);
    GVOTE_CHECK_LAUNCH();
  }
  hipLaunchKernelGGL((score_emit_kernel<DK, NT>), dim3(grid_wg * tab.emit_split), dim3(kThreads), 0, st, tab);
  GVOTE_CHECK_LAUNCH();
  return GVOTE_OK;
}

int emit_split_of(int chunk_keys) { return chunk_keys > kMaxEmitKeys ? 2 : 1; }

int g_spin_limit = 1 << 22;     // polls of a finished pass-1 wave waiting for its workgroup before it gives up

}  // namespace

int set_hist_spin_limit(int polls) {
  const int old = g_spin_limit;
  g_spin_limit = polls < 0 ? (1 << 22) : polls;
  return old;
}

bool fast_path_ok(const gvote_shape *sh, int S, int mode, float p) {
  const int NQ = S * (sh->n_q_heads / sh->n_kv_heads);
  if (sh->dtype != GVOTE_BF16 || (sh->head_dim != 64 && sh->head_dim != 128) || NQ < 1) return false;
  return mode == GVOTE_SELECT_TOPK || (mode == GVOTE_SELECT_TOPP && p < 1.0f);
}

FastPlan plan_fast(const gvote_shape *sh, const gvote_item *items, int n_items, int S) {
  FastPlan pl;
  const int NQ = S * (sh->n_q_heads / sh->n_kv_heads);
  size_t max_slots = 0, max_rows = 0, max_tiles = 0, max_sub = 0;
  for (int b0 = 0; b0 < n_items; b0 += kMaxItems) {
    const int nb = n_items - b0 < kMaxItems ? n_items - b0 : kMaxItems;
    const int ck = pick_chunk_keys(sh, items + b0, nb);
    size_t slots = 0, tiles = 0;
    for (int i = 0; i < nb; ++i) {
      const size_t sub = (size_t)ceil_div(items[b0 + i].L, ck) * emit_split_of(ck) * 2 * kWaves;
      if (sub > max_sub) max_sub = sub;
      slots += (size_t)sh->n_kv_heads * ceil_div(items[b0 + i].L, ck);
      tiles += (size_t)sh->n_kv_heads * ((items[b0 + i].L + 31) / 32);
    }
    if (slots > max_slots) max_slots = slots;
    if (tiles > max_tiles) max_tiles = tiles;
    const size_t rows = (size_t)nb * S * sh->n_q_heads;
    if (rows > max_rows) max_rows = rows;
  }
  pl.off_max = 256;   // the first 256 bytes hold the fallback-row counter
  pl.off_top = pl.off_max + align_up(max_slots * NQ * sizeof(float), 256);
  pl.off_hist = pl.off_top + align_up(max_slots * NQ * sizeof(int), 256);
  pl.off_info = pl.off_hist + align_up(max_slots * NQ * kBins * sizeof(float), 256);
  pl.off_cnt = pl.off_info + align_up(max_rows * sizeof(RowInfo), 256);
  pl.off_cands = pl.off_cnt + align_up(max_rows * max_sub * sizeof(int), 256);
  pl.off_tmax = pl.off_cands + align_up(max_rows * max_sub * kSubCap * sizeof(uint2), 256);
  pl.off_list = pl.off_tmax + align_up(max_tiles * NQ * sizeof(short), 256);
  pl.off_ovfc = pl.off_list + align_up(max_rows * sizeof(int), 256);
  pl.off_ovf = pl.off_ovfc + align_up(max_rows * sizeof(int), 256);
  pl.ws_bytes = pl.off_ovf + align_up(max_rows * kOvfCap * sizeof(uint2), 256);
  return pl;
}

gvote_status launch_score_fast(const gvote_shape *sh, const gvote_item *items, int n_items, int S, const void *q,
                               float p, int mode, const int *k_per_row, uint32_t *rowmask, float *row_max,
                               float *row_sum, void *ws, hipStream_t st) {
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
    tab.spin_limit = g_spin_limit;
    tab.q = q; tab.k_per_row = k_per_row; tab.mode = mode;
    tab.rowmask = rowmask; tab.row_max = row_max; tab.row_sum = row_sum;
    tab.n_fallback = reinterpret_cast<int *>(wsb);
    tab.n_list = reinterpret_cast<int *>(wsb) + 1;
    tab.n_refine = reinterpret_cast<int *>(wsb) + 8;
    tab.row_list = reinterpret_cast<int *>(wsb + pl.off_list);
    tab.ovf_cnt = reinterpret_cast<int *>(wsb + pl.off_ovfc);
    tab.ovf = reinterpret_cast<uint2 *>(wsb + pl.off_ovf);
    tab.part_max = reinterpret_cast<float *>(wsb + pl.off_max);
    tab.part_top = reinterpret_cast<int *>(wsb + pl.off_top);
    tab.tile_bin = reinterpret_cast<short *>(wsb + pl.off_tmax);
    tab.part_hist = reinterpret_cast<uint32_t *>(wsb + pl.off_hist);
    tab.info = reinterpret_cast<RowInfo *>(wsb + pl.off_info);
    tab.cand_cnt = reinterpret_cast<int *>(wsb + pl.off_cnt);
    tab.cands = reinterpret_cast<uint2 *>(wsb + pl.off_cands);
    int wg = 0, part = 0, most_chunks = 0;
    long long tmax0 = 0;
    for (int i = 0; i < nb; ++i) {
      const gvote_item &g = items[b0 + i];
      FastItem &f = tab.it[i];
      f.k = g.k; f.tok_stride = g.kv_tok_stride; f.head_stride = g.kv_head_stride;
      f.mask_off = mask_off; f.L = g.L; f.W = (g.L + 31) / 32;
      f.n_chunks = ceil_div(g.L, tab.chunk_keys);
      if (f.n_chunks > most_chunks) most_chunks = f.n_chunks;
      f.wg0 = wg; f.part0 = part; f.pad = 0; f.tmax0 = tmax0;
      tmax0 += (long long)sh->n_kv_heads * f.W * tab.NQ;
      wg += sh->n_kv_heads * f.n_chunks * tab.NQB;
      part += sh->n_kv_heads * f.n_chunks;
      mask_off += (long long)tab.rows_per_item * f.W;
    }
    tab.emit_split = emit_split_of(tab.chunk_keys);
    tab.sub_per_row = most_chunks * tab.emit_split * 2 * kWaves;
    tab.n_slots = part;
    const int grid_wg = tab.NQB == 1 ? wg : ceil_div(part, 8) * 8 * tab.NQB;
    const int rows = nb * tab.rows_per_item;
    const bool topk = mode == GVOTE_SELECT_TOPK;
    gvote_status lst;
    const bool nt = tab.NQB == 1;
    if (sh->head_dim == 128) lst = nt ? launch_passes<128, true>(tab, grid_wg, rows, topk, st) : launch_passes<128, false>(tab, grid_wg, rows, topk, st);
    else lst = nt ? launch_passes<64, true>(tab, grid_wg, rows, topk, st) : launch_passes<64, false>(tab, grid_wg, rows, topk, st);
    if (lst != GVOTE_OK) return lst;
    hipLaunchKernelGGL((resolve_kernel<256, false>), dim3(ceil_div(rows, 4)), dim3(256), 0, st, tab, rows);
    GVOTE_CHECK_LAUNCH();
    hipLaunchKernelGGL((resolve_kernel<kCandCap, true>), dim3(rows), dim3(64), 0, st, tab, rows);
    GVOTE_CHECK_LAUNCH();
    // rows the histogram could not settle are redone exactly
    gvote_status stt = launch_select_rows_general(sh, items + b0, nb, b0, S, q, p, mode, k_per_row, rowmask,
                                                  batch_mask_off0, row_max, row_sum, tab.row_list, tab.n_list,
                                                  tab.n_fallback, reinterpret_cast<float *>(wsb + pl.ws_bytes),
                                                  general_cache_bytes(items, n_items), st);
    if (stt != GVOTE_OK) return stt;
  }
  return GVOTE_OK;
}

}  // namespace gvote
