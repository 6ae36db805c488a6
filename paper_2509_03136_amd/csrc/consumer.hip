// Consumer side of the compressed cache (paper Sec. 3.4: a non-uniform, per-head cache read through a
// variable-length attention interface; Eq. (1)-(2)), and the attention-overlap diagnostic of Sec. 3.3.
//
//   decode_attention   one decode query per head against the packed rows of its KV head:
//                      softmax(q K^T / sqrt(d_k)) V.  The packed rows of a head are split over several
//                      workgroups (so that few heads still fill the chip); each serves the G query heads of
//                      the group over its share, so every packed K/V row is read once (16 bytes per lane,
//                      a key row by d_k*elem/16 neighbouring lanes); results are merged across the wave by
//                      shuffles, across the workgroup through LDS, across the shares by a small merge kernel
//                      through their log-sum-exp.  Memory-bound (2 * B * d_k * elem bytes per KV head).
//                      bf16 with d_k 64 or 128 and up to 16 heads per KV head: logits of 32-row tiles on the
//                      matrix cores, one rescale per tile (decode_attention_mfma_kernel); everything else:
//                      vector units, online softmax per row step (decode_attention_kernel).
//   attention_overlap  how much of a REAL query's attention falls on the key set a synthetic row chose:
//                      per (item, query head) the real query's logits over all L keys (kept in the
//                      workspace), their softmax, and for every sample s the weight inside row (s, h)'s mask.
#include "gvote_internal.hpp"

namespace gvote {

namespace {

constexpr int kGMax = 8;    // query heads of a group handled per sweep over the packed rows
constexpr int kRowsInFlight = 4;   // row steps a lane loads before it consumes them

struct DecodeArgs {
  const void *q, *k_out, *v_out;
  const long long *offsets;
  void *out;
  float *lse;
  float *part;              // workspace: [item * H_q + h][split][d_k + 2]: un-normalised output, row maximum, weight sum
  int n_q_heads, n_kv_heads, head_dim, n_splits;
  float scale;              // log2(e) / sqrt(d_k): logits are kept in log2 units, weights are powers of two
};

// grid (item * H_kv + kv head, split): one workgroup serves the G query heads of the group over ITS SHARE of the
// head's packed rows (several workgroups per head keep the whole chip streaming even with few heads); the shares
// are merged by decode_merge_kernel through their log-sum-exp.
template <typename T>
__global__ __launch_bounds__(256) void decode_attention_kernel(const DecodeArgs a) {
  constexpr int NV = Vec16<T>::N;
  const int dk = a.head_dim;
  const int ppr = dk / NV;                       // lanes per row (power of two, <= 64: checked by the host)
  const int rps = 64 / ppr;                      // rows per wave step
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int piece = lane % ppr, rs = lane / ppr;
  const int hh = blockIdx.x;                     // item * H_kv + kv head
  const int split = blockIdx.y;
  const int item = hh / a.n_kv_heads, kvh = hh - item * a.n_kv_heads;
  const int G = a.n_q_heads / a.n_kv_heads;
  const long long lo_h = a.offsets[hh], n_h = a.offsets[hh + 1] - lo_h;
  const long long lo = lo_h + n_h * split / a.n_splits, hi = lo_h + n_h * (split + 1) / a.n_splits;
  const T *kb = reinterpret_cast<const T *>(a.k_out);
  const T *vb = reinterpret_cast<const T *>(a.v_out);
  __shared__ float part[4][kGMax][256 + 2];      // per wave: acc[d_k], m, l of every head of the sweep

  for (int g0 = 0; g0 < G; g0 += kGMax) {
    const int ng = min(kGMax, G - g0);
    float qv[kGMax][NV], m[kGMax], l[kGMax], acc[kGMax][NV];
#pragma unroll
    for (int g = 0; g < kGMax; ++g) {
      m[g] = -INFINITY;
      l[g] = 0.f;
#pragma unroll
      for (int i = 0; i < NV; ++i) { acc[g][i] = 0.f; qv[g][i] = 0.f; }
      if (g < ng) {
        const T *qrow = reinterpret_cast<const T *>(a.q) + ((size_t)item * a.n_q_heads + kvh * G + g0 + g) * dk;
        Vec16<T>::load(qrow + piece * NV, qv[g]);
      }
    }
    // kRowsInFlight row steps are loaded (K and V, 16 bytes per lane each) before any is consumed
    for (long long r0 = lo + (long long)wave * rps; r0 < hi; r0 += 4 * rps * kRowsInFlight) {
      float kv[kRowsInFlight][NV], vv[kRowsInFlight][NV];
#pragma unroll
      for (int u = 0; u < kRowsInFlight; ++u) {
        const long long r = r0 + (long long)u * 4 * rps + rs;
        const long long rc = r < hi ? r : hi - 1;          // in bounds (hi > lo here); the contribution is dropped
        Vec16Stream<T>::load(kb + rc * dk + piece * NV, kv[u]);
        Vec16Stream<T>::load(vb + rc * dk + piece * NV, vv[u]);
      }
#pragma unroll
      for (int u = 0; u < kRowsInFlight; ++u) {
        const bool valid = r0 + (long long)u * 4 * rps + rs < hi;
#pragma unroll
        for (int g = 0; g < kGMax; ++g) {
          if (g < ng) {
            float s = 0.f;
#pragma unroll
            for (int i = 0; i < NV; ++i) s = fmaf(qv[g][i], kv[u][i], s);
            for (int off = ppr >> 1; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
            s *= a.scale;
            if (valid) {
              const float mn = fmaxf(m[g], s);
              const float corr = __builtin_amdgcn_exp2f(m[g] - mn), pw = __builtin_amdgcn_exp2f(s - mn);     // 2^(-inf) = 0 on the first row
              l[g] = l[g] * corr + pw;
#pragma unroll
              for (int i = 0; i < NV; ++i) acc[g][i] = fmaf(acc[g][i], corr, pw * vv[u][i]);
              m[g] = mn;
            }
          }
        }
      }
    }
    // merge the row slots of the wave (lanes with the same piece), then the four waves
#pragma unroll
    for (int g = 0; g < kGMax; ++g) {
      if (g < ng) {
        for (int off = ppr; off < 64; off <<= 1) {
          const float mo = __shfl_xor(m[g], off, 64), lo2 = __shfl_xor(l[g], off, 64);
          const float mn = fmaxf(m[g], mo);
          const float ca = mn == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(m[g] - mn), cb = mn == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(mo - mn);
          l[g] = l[g] * ca + lo2 * cb;
#pragma unroll
          for (int i = 0; i < NV; ++i) acc[g][i] = acc[g][i] * ca + __shfl_xor(acc[g][i], off, 64) * cb;
          m[g] = mn;
        }
        if (rs == 0) {
#pragma unroll
          for (int i = 0; i < NV; ++i) part[wave][g][piece * NV + i] = acc[g][i];
          if (piece == 0) { part[wave][g][256] = m[g]; part[wave][g][257] = l[g]; }
        }
      }
    }
    __syncthreads();
    for (int o = threadIdx.x; o < ng * (dk + 2); o += 256) {
      const int g = o / (dk + 2), ch = o - g * (dk + 2);
      float mn = -INFINITY;
      for (int w = 0; w < 4; ++w) mn = fmaxf(mn, part[w][g][256]);
      float val;
      if (ch == dk) {
        val = mn;
      } else {
        val = 0.f;
        for (int w = 0; w < 4; ++w) {
          const float cw = part[w][g][256] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(part[w][g][256] - mn);
          val = fmaf(part[w][g][ch < dk ? ch : 257], cw, val);
        }
      }
      const size_t row = (size_t)item * a.n_q_heads + kvh * G + g0 + g;
      a.part[(row * a.n_splits + split) * (dk + 2) + ch] = val;      // ch < dk: numerator; dk: maximum; dk + 1: weight sum
    }
    __syncthreads();
  }
}

// ---- bf16, d_k 64 or 128, G <= 16: the logits of 32 packed rows against the group's query heads come from the
// matrix cores.  Same grid, shares and partial results as decode_attention_kernel.  Per wave and 32-row tile:
//   K rows (coalesced 16-byte lanes, non-temporal) -> wave-private XOR-swizzled LDS tile -> A operand of
//   v_mfma_f32_32x32x16_bf16, the B operand holds the query heads as columns (columns >= G are zero), so lane
//   (col, hf) ends up with the logits of head `col` for 16 of the 32 rows;
//   the lanes of the G heads take the tile maximum, rescale their running sums once per TILE (not per row) and
//   leave the 32 x G weights and the G rescale factors in LDS;
//   the V rows stay in registers as they were loaded (a lane owns 8 channels of every fourth or eighth row):
//   acc[g][8] = acc[g][8] * corr[g] + sum_rows p[row][g] * v[row][8] on the vector units, the weights coming
//   from LDS as broadcast reads.
// The next tile's K and V rows are in flight while the current one is processed.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));
__device__ __forceinline__ int tile_row_of(int r, int hf) { return 8 * (r >> 2) + 4 * hf + (r & 3); }   // C layout of the 32x32 MFMA

template <int DK, int GP>
__global__ __launch_bounds__(256) void decode_attention_mfma_kernel(const DecodeArgs a) {
  constexpr int KS = DK / 16, PPR = DK / 8, RPL = 64 / PPR, LOADS = 32 / RPL;
  constexpr int TILE_BYTES = 32 * DK * 2;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, hf = lane >> 5;
  const int piece = lane % PPR, sub = lane / PPR;
  const int hh = blockIdx.x, split = blockIdx.y;
  const int item = hh / a.n_kv_heads, kvh = hh - item * a.n_kv_heads;
  const int G = a.n_q_heads / a.n_kv_heads;
  const long long lo_h = a.offsets[hh], n_h = a.offsets[hh + 1] - lo_h;
  const long long lo = lo_h + n_h * split / a.n_splits, hi = lo_h + n_h * (split + 1) / a.n_splits;
  const char *kb = reinterpret_cast<const char *>(a.k_out);
  const char *vb = reinterpret_cast<const char *>(a.v_out);
  __shared__ __align__(16) unsigned char ktile[4][TILE_BYTES];
  __shared__ __align__(16) float pw[4][32][GP];       // weights of the tile: [row][head]
  __shared__ __align__(16) float corr_s[4][GP];
  __shared__ float part[4][GP][DK + 2];               // per wave: acc[d_k], m, l of every head

  // B operand: query head `col` of the group (zero columns beyond G)
  bf16x8 bq[KS];
  {
    const bf16_t *qrow = reinterpret_cast<const bf16_t *>(a.q) + ((size_t)item * a.n_q_heads + kvh * G + (col < G ? col : 0)) * DK + 8 * hf;
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) {
      uint4 raw = make_uint4(0, 0, 0, 0);
      if (col < G) raw = *reinterpret_cast<const uint4 *>(qrow + 16 * ks);
      bq[ks] = __builtin_bit_cast(bf16x8, raw);
    }
  }
  float m_run = -INFINITY, l_run = 0.f;      // of head `col`, over this lane's 16 rows of every tile (the two halves share m_run)
  float acc[GP][8];
#pragma unroll
  for (int g = 0; g < GP; ++g)
#pragma unroll
    for (int i = 0; i < 8; ++i) acc[g][i] = 0.f;

  const long long n_rows = hi - lo;
  const long long n_tiles = (n_rows + 31) >> 5;
  auto fetch = [&](u32x4_t(&pk)[LOADS], u32x4_t(&pv)[LOADS], long long tile) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < LOADS; ++j) {
      long long r = lo + tile * 32 + j * RPL + sub;
      r = r < hi ? r : hi - 1;               // in bounds (hi > lo here); the row's weight is forced to zero
      pk[j] = load_stream16(kb + (r * DK + piece * 8) * 2);
      pv[j] = load_stream16(vb + (r * DK + piece * 8) * 2);
    }
  };
  unsigned char *kt = ktile[wave];
  if (wave < n_tiles) {
    u32x4_t pk[LOADS], pv[LOADS], vcur[LOADS];
    fetch(pk, pv, wave);
    for (long long tile = wave; tile < n_tiles; tile += 4) {
#pragma unroll
      for (int j = 0; j < LOADS; ++j) {
        const int row = j * RPL + sub;
        *reinterpret_cast<u32x4_t *>(kt + (row * PPR + (piece ^ (row & (PPR - 1)))) * 16) = pk[j];
        vcur[j] = pv[j];
      }
      {
        const long long tn = tile + 4 < n_tiles ? tile + 4 : tile;     // (the last tile is fetched again: no conditional load)
        fetch(pk, pv, tn);
      }
      __builtin_amdgcn_wave_barrier();
      floatx16 c;
#pragma unroll
      for (int r = 0; r < 16; ++r) c[r] = 0.f;
#pragma unroll
      for (int ks = 0; ks < KS; ++ks) {
        const int phys = (2 * ks + hf) ^ (col & (PPR - 1));
        const bf16x8 ak = *reinterpret_cast<const bf16x8 *>(kt + (col * PPR + phys) * 16);     // row `col` of the tile
        c = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ak, bq[ks], c, 0, 0, 0);
      }
      // softmax bookkeeping of head `col` (all lanes run it; only columns < G are looked at afterwards)
      const int valid = (int)((hi - lo - tile * 32) < 32 ? (hi - lo - tile * 32) : 32);
      float mt = -INFINITY;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        c[r] = tile_row_of(r, hf) < valid ? c[r] * a.scale : -INFINITY;
        mt = fmaxf(mt, c[r]);
      }
      mt = fmaxf(mt, __shfl_xor(mt, 32, 64));
      const float mn = fmaxf(m_run, mt);                      // finite: row 0 of a tile always exists
      const float corr = __builtin_amdgcn_exp2f(m_run - mn);   // 2^(-inf) = 0 on the first tile
      float ls = 0.f;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const float pr = __builtin_amdgcn_exp2f(c[r] - mn);
        ls += pr;
        if (col < GP) pw[wave][tile_row_of(r, hf)][col] = pr;
      }
      l_run = l_run * corr + ls;
      m_run = mn;
      if (lane < GP) corr_s[wave][lane] = corr;
      __builtin_amdgcn_wave_barrier();
      // output update: this lane's 8 channels of its rows
      float cg[GP];
#pragma unroll
      for (int g4 = 0; g4 < GP; g4 += 4) {
        const float4 t = *reinterpret_cast<const float4 *>(&corr_s[wave][g4]);
        cg[g4] = t.x; cg[g4 + 1] = t.y; cg[g4 + 2] = t.z; cg[g4 + 3] = t.w;
      }
#pragma unroll
      for (int g = 0; g < GP; ++g)
#pragma unroll
        for (int i = 0; i < 8; ++i) acc[g][i] *= cg[g];
#pragma unroll
      for (int j = 0; j < LOADS; ++j) {
        const int row = j * RPL + sub;
        float vv[8];
        vv[0] = __uint_as_float(vcur[j].x << 16); vv[1] = __uint_as_float(vcur[j].x & 0xFFFF0000u);
        vv[2] = __uint_as_float(vcur[j].y << 16); vv[3] = __uint_as_float(vcur[j].y & 0xFFFF0000u);
        vv[4] = __uint_as_float(vcur[j].z << 16); vv[5] = __uint_as_float(vcur[j].z & 0xFFFF0000u);
        vv[6] = __uint_as_float(vcur[j].w << 16); vv[7] = __uint_as_float(vcur[j].w & 0xFFFF0000u);
#pragma unroll
        for (int g4 = 0; g4 < GP; g4 += 4) {
          const float4 t = *reinterpret_cast<const float4 *>(&pw[wave][row][g4]);
          const float pg[4] = {t.x, t.y, t.z, t.w};
#pragma unroll
          for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int i = 0; i < 8; ++i) acc[g4 + q][i] = fmaf(pg[q], vv[i], acc[g4 + q][i]);
        }
      }
      __builtin_amdgcn_wave_barrier();
    }
  }
  // the wave's result: sum the row subsets (lanes with the same piece), the two halves of l
  l_run += __shfl_xor(l_run, 32, 64);
#pragma unroll
  for (int g = 0; g < GP; ++g) {
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      float x = acc[g][i];
      for (int off = PPR; off < 64; off <<= 1) x += __shfl_xor(x, off, 64);
      acc[g][i] = x;
    }
    if (sub == 0 && g < G) {
#pragma unroll
      for (int i = 0; i < 8; ++i) part[wave][g][piece * 8 + i] = acc[g][i];
    }
  }
  if (lane < G) { part[wave][lane][DK] = m_run; part[wave][lane][DK + 1] = l_run; }
  __syncthreads();
  for (int o = threadIdx.x; o < G * (DK + 2); o += 256) {
    const int g = o / (DK + 2), ch = o - g * (DK + 2);
    float mn = -INFINITY;
    for (int w = 0; w < 4; ++w) mn = fmaxf(mn, part[w][g][DK]);
    float val;
    if (ch == DK) {
      val = mn;
    } else {
      val = 0.f;
      for (int w = 0; w < 4; ++w) {
        const float cw = part[w][g][DK] == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(part[w][g][DK] - mn);
        val = fmaf(part[w][g][ch < DK ? ch : DK + 1], cw, val);
      }
    }
    const size_t row = (size_t)item * a.n_q_heads + kvh * G + g;
    a.part[(row * a.n_splits + split) * (DK + 2) + ch] = val;      // ch < d_k: numerator; d_k: maximum; d_k + 1: weight sum
  }
}

// one workgroup per (item, query head): out = sum_s e^(m_s - m) num_s / sum_s e^(m_s - m) l_s
template <typename T>
__global__ __launch_bounds__(256) void decode_merge_kernel(const DecodeArgs a) {
  const size_t row = blockIdx.x;
  const int dk = a.head_dim;
  const float *p = a.part + row * a.n_splits * (dk + 2);
  float mn = -INFINITY;
  for (int s = 0; s < a.n_splits; ++s) mn = fmaxf(mn, p[s * (dk + 2) + dk]);
  float den = 0.f;
  for (int s = 0; s < a.n_splits; ++s) {
    const float ms = p[s * (dk + 2) + dk];
    den = fmaf(p[s * (dk + 2) + dk + 1], ms == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms - mn), den);
  }
  for (int ch = threadIdx.x; ch < dk; ch += 256) {
    float num = 0.f;
    for (int s = 0; s < a.n_splits; ++s) {
      const float ms = p[s * (dk + 2) + dk];
      num = fmaf(p[s * (dk + 2) + ch], ms == -INFINITY ? 0.f : __builtin_amdgcn_exp2f(ms - mn), num);
    }
    reinterpret_cast<T *>(a.out)[row * dk + ch] = from_f32<T>(den > 0.f ? num / den : 0.f);
  }
  if (threadIdx.x == 0 && a.lse) a.lse[row] = den > 0.f ? (mn + log2f(den)) * 0.69314718055994530942f : -INFINITY;
}

// ---------------------------------------------------------------- attention overlap
struct OverlapItem {
  const void *k;
  long long tok_stride, head_stride, mask_off, cache_off;
  int L, W;
};
struct OverlapTable {
  int n_items, S, n_q_heads, n_kv_heads, head_dim, item0;
  double scale;
  const void *q_real;          // [n_items_call][H_q][d_k]
  const uint32_t *rowmask;
  float *overlap;              // [n_items_call][S][H_q]
  float *cache;                // workspace: the real query's logits, one slice per (item, head)
  OverlapItem it[kMaxItems];
};

template <typename T>
__global__ __launch_bounds__(256) void attention_overlap_kernel(const OverlapTable tab) {
  constexpr int NV = Vec16<T>::N;
  typedef typename Acc<T>::type acc_t;
  const int it = blockIdx.x / tab.n_q_heads, h = blockIdx.x - it * tab.n_q_heads;
  const OverlapItem I = tab.it[it];
  const int kvh = h / (tab.n_q_heads / tab.n_kv_heads);
  const int dk = tab.head_dim, L = I.L;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  __shared__ float q_s[256];
  __shared__ float red[4];
  const T *qrow = reinterpret_cast<const T *>(tab.q_real) + ((size_t)(tab.item0 + it) * tab.n_q_heads + h) * dk;
  if (tid < dk) q_s[tid] = to_f32<T>(qrow[tid]);
  __syncthreads();
  float *cache = tab.cache + I.cache_off + (long long)h * ((L + 63) / 64 * 64);
  const T *kbase = reinterpret_cast<const T *>(I.k) + (long long)kvh * I.head_stride;
  const int ppr = dk / NV;
  int lpk = 1;
  while (lpk < ppr) lpk <<= 1;
  const int kpi = 256 / lpk, slot = tid / lpk, piece = tid - slot * lpk;
  auto block_max = [&](float v) {
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    if (lane == 0) red[wave] = v;
    __syncthreads();
    v = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    __syncthreads();
    return v;
  };
  auto block_sum = [&](float v) {
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    if (lane == 0) red[wave] = v;
    __syncthreads();
    v = red[0] + red[1] + red[2] + red[3];
    __syncthreads();
    return v;
  };
  // logits of the real query (a key row is read by lpk neighbouring lanes), kept in the workspace
  float m = -INFINITY;
  for (int t0 = 0; t0 < L; t0 += kpi) {
    const int t = t0 + slot;
    acc_t acc = 0;
    if (piece < ppr && t < L) {
      float kv[NV];
      Vec16<T>::load(kbase + (long long)t * I.tok_stride + piece * NV, kv);
#pragma unroll
      for (int i = 0; i < NV; ++i) acc = fma((acc_t)q_s[piece * NV + i], (acc_t)kv[i], acc);
    }
    for (int off = lpk >> 1; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (piece == 0 && t < L) {
      const float lg = (float)(acc * (acc_t)tab.scale);
      cache[t] = lg;
      m = fmaxf(m, lg);
    }
  }
  m = block_max(m);
  __threadfence_block();
  __syncthreads();
  float z = 0.f;
  for (int t = tid; t < L; t += 256) z += expf(cache[t] - m);
  z = block_sum(z);
  for (int s = 0; s < tab.S; ++s) {
    const uint32_t *mrow = tab.rowmask + I.mask_off + (long long)(s * tab.n_q_heads + h) * I.W;
    float w = 0.f;
    for (int t = tid; t < L; t += 256)
      if ((mrow[t >> 5] >> (t & 31)) & 1u) w += expf(cache[t] - m);
    w = block_sum(w);
    if (tid == 0) tab.overlap[((size_t)(tab.item0 + it) * tab.S + s) * tab.n_q_heads + h] = w / z;
  }
}

}  // namespace

size_t overlap_ws_bytes(const gvote_shape *sh, const gvote_item *items, int n_items) {
  size_t worst = 0;
  for (int b0 = 0; b0 < n_items; b0 += kMaxItems) {
    const int nb = n_items - b0 < kMaxItems ? n_items - b0 : kMaxItems;
    size_t f = 0;
    for (int i = 0; i < nb; ++i) f += (size_t)sh->n_q_heads * ((items[b0 + i].L + 63) / 64 * 64);
    if (f > worst) worst = f;
  }
  return worst * sizeof(float);
}

int decode_splits(const gvote_shape *sh, int n_items) {
  // about two workgroups per CU over the call (measured on 256 heads of ~4000 rows: 256..512 workgroups 0.095 ms,
  // 1024 0.099, 2048 0.111, 4096 0.136), at most 64 shares per head
  const int heads = n_items * sh->n_kv_heads;
  int s = (512 + heads - 1) / heads;
  return s < 1 ? 1 : (s > 64 ? 64 : s);
}

size_t decode_ws_bytes(const gvote_shape *sh, int n_items) {
  return (size_t)n_items * sh->n_q_heads * decode_splits(sh, n_items) * (sh->head_dim + 2) * sizeof(float);
}

gvote_status launch_decode_attention(const gvote_shape *sh, int n_items, const void *q, const void *k_out,
                                     const void *v_out, const long long *offsets, void *out, float *lse, void *ws,
                                     hipStream_t st) {
  DecodeArgs a;
  a.q = q; a.k_out = k_out; a.v_out = v_out; a.offsets = offsets; a.out = out; a.lse = lse;
  a.part = reinterpret_cast<float *>(ws);
  a.n_q_heads = sh->n_q_heads; a.n_kv_heads = sh->n_kv_heads; a.head_dim = sh->head_dim;
  a.n_splits = decode_splits(sh, n_items);
  a.scale = (float)(1.44269504088896340736 / sqrt((double)sh->head_dim));
  const dim3 grid(n_items * sh->n_kv_heads, a.n_splits);
  const dim3 gridm(n_items * sh->n_q_heads);
  if (sh->dtype == GVOTE_F32) {
    hipLaunchKernelGGL(decode_attention_kernel<float>, grid, dim3(256), 0, st, a);
    GVOTE_CHECK_LAUNCH();
    hipLaunchKernelGGL(decode_merge_kernel<float>, gridm, dim3(256), 0, st, a);
  } else {
    const int G = sh->n_q_heads / sh->n_kv_heads;
    const bool mfma = (sh->head_dim == 64 || sh->head_dim == 128) && G <= 16;
    if (!mfma) hipLaunchKernelGGL(decode_attention_kernel<bf16_t>, grid, dim3(256), 0, st, a);
    else if (sh->head_dim == 128 && G <= 4) hipLaunchKernelGGL((decode_attention_mfma_kernel<128, 4>), grid, dim3(256), 0, st, a);
    else if (sh->head_dim == 128 && G <= 8) hipLaunchKernelGGL((decode_attention_mfma_kernel<128, 8>), grid, dim3(256), 0, st, a);
    else if (sh->head_dim == 128) hipLaunchKernelGGL((decode_attention_mfma_kernel<128, 16>), grid, dim3(256), 0, st, a);
    else if (G <= 4) hipLaunchKernelGGL((decode_attention_mfma_kernel<64, 4>), grid, dim3(256), 0, st, a);
    else if (G <= 8) hipLaunchKernelGGL((decode_attention_mfma_kernel<64, 8>), grid, dim3(256), 0, st, a);
    else hipLaunchKernelGGL((decode_attention_mfma_kernel<64, 16>), grid, dim3(256), 0, st, a);
    GVOTE_CHECK_LAUNCH();
    hipLaunchKernelGGL(decode_merge_kernel<bf16_t>, gridm, dim3(256), 0, st, a);
  }
  GVOTE_CHECK_LAUNCH();
  return GVOTE_OK;
}

gvote_status launch_attention_overlap(const gvote_shape *sh, const gvote_item *items, int n_items, int S,
                                      const void *q_real, const uint32_t *rowmask, float *overlap, void *ws,
                                      hipStream_t st) {
  long long mask_off = 0;
  for (int b0 = 0; b0 < n_items; b0 += kMaxItems) {
    const int nb = n_items - b0 < kMaxItems ? n_items - b0 : kMaxItems;
    OverlapTable tab;
    tab.n_items = nb; tab.S = S; tab.n_q_heads = sh->n_q_heads; tab.n_kv_heads = sh->n_kv_heads;
    tab.head_dim = sh->head_dim; tab.item0 = b0; tab.scale = 1.0 / sqrt((double)sh->head_dim);
    tab.q_real = q_real; tab.rowmask = rowmask; tab.overlap = overlap; tab.cache = reinterpret_cast<float *>(ws);
    long long cache_off = 0;
    for (int i = 0; i < nb; ++i) {
      const gvote_item &g = items[b0 + i];
      OverlapItem &o = tab.it[i];
      o.k = g.k; o.tok_stride = g.kv_tok_stride; o.head_stride = g.kv_head_stride;
      o.L = g.L; o.W = (g.L + 31) / 32; o.mask_off = mask_off; o.cache_off = cache_off;
      mask_off += (long long)S * sh->n_q_heads * o.W;
      cache_off += (long long)sh->n_q_heads * ((g.L + 63) / 64 * 64);
    }
    const dim3 grid(nb * sh->n_q_heads);
    if (sh->dtype == GVOTE_F32)
      hipLaunchKernelGGL(attention_overlap_kernel<float>, grid, dim3(256), 0, st, tab);
    else
      hipLaunchKernelGGL(attention_overlap_kernel<bf16_t>, grid, dim3(256), 0, st, tab);
    GVOTE_CHECK_LAUNCH();
  }
  return GVOTE_OK;
}

}  // namespace gvote
