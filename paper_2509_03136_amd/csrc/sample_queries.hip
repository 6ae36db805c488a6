// Stage 2 - synthetic future queries (paper Sec. 3.2 Step 3; Alg. 1: the Gaussian draw
// "H~ ~ N(mu, diag sigma^2)", "AverageCosSin(n_f)" and "Q~ = RoPE(H~ W_q, P)").
//
//   sample_hidden   Philox4x32-10 (counter = draw index, so any thread regenerates any element)
//                   -> Box-Muller -> mu + sigma z, rounded to the storage type.  S*d values per
//                   item (KBs), so it is generated once instead of once per GEMM workgroup.
//   project_mfma    bf16: the [S, d] x [d, H_q d_k] product is a skinny GEMM whose cost is the one
//                   read of W_q; W_q rows are the A operand of v_mfma_f32_32x32x16_bf16 straight
//                   from global memory (each lane owns 64 contiguous bytes of one row per k-step),
//                   the sampled states are the B operand from LDS.  Split along k so that even a
//                   single item fills the chip; partial sums are reduced in a fixed order.
//   project_generic any storage type, plain FMA (the fp32 configuration).
//   rope_finalize   k-split reduction + bias + rotation by the averaged cos/sin (computed in fp64
//                   on the device: the angle pos * omega needs more than fp32 at 128k) + rounding.
#include "gvote_internal.hpp"

namespace gvote {

namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float floatx16 __attribute__((ext_vector_type(16)));

// ---- Philox4x32-10 (Salmon et al., SC'11): ten rounds, Weyl key schedule
__device__ __forceinline__ void philox4x32_10(uint32_t (&c)[4], uint32_t k0, uint32_t k1) {
  constexpr uint32_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u, W0 = 0x9E3779B9u, W1 = 0xBB67AE85u;
#pragma unroll
  for (int r = 0; r < 10; ++r) {
    const uint32_t hi0 = __umulhi(M0, c[0]), lo0 = M0 * c[0];
    const uint32_t hi1 = __umulhi(M1, c[2]), lo1 = M1 * c[2];
    const uint32_t n0 = hi1 ^ c[1] ^ k0, n2 = hi0 ^ c[3] ^ k1;
    c[0] = n0; c[1] = lo1; c[2] = n2; c[3] = lo0;
    k0 += W0; k1 += W1;
  }
}

// u = ((x >> 9) + 1/2) 2^-23 is exact in fp32 and lies strictly inside (0, 1)
__device__ __forceinline__ float u01(uint32_t x) { return ((float)(x >> 9) + 0.5f) * 0x1.0p-23f; }

__device__ __forceinline__ void box_muller(uint32_t xa, uint32_t xb, float &z_even, float &z_odd) {
  const float r = sqrtf(-2.0f * logf(u01(xa)));
  float sn, cs;
  sincospif(2.0f * u01(xb), &sn, &cs);   // angle 2 pi u_b, argument exact
  z_even = r * cs;
  z_odd = r * sn;
}

__global__ __launch_bounds__(256) void philox_u32_kernel(unsigned long long seed, unsigned long long sid, long long n,
                                                         uint32_t *out) {
  const long long blk = (long long)blockIdx.x * 256 + threadIdx.x;
  if (blk * 4 >= n) return;
  uint32_t c[4] = {(uint32_t)blk, (uint32_t)((unsigned long long)blk >> 32), (uint32_t)sid, (uint32_t)(sid >> 32)};
  philox4x32_10(c, (uint32_t)seed, (uint32_t)(seed >> 32));
#pragma unroll
  for (int i = 0; i < 4; ++i)
    if (blk * 4 + i < n) out[blk * 4 + i] = c[i];
}

template <typename T>
__global__ __launch_bounds__(256) void sample_hidden_kernel(const SampleTable tab) {
  const int it = blockIdx.y;
  const long long blk = (long long)blockIdx.x * 256 + threadIdx.x;
  const long long e0 = blk * 4;
  if (e0 >= (long long)tab.S * tab.d) return;
  const SampleItem I = tab.it[it];
  uint32_t c[4] = {(uint32_t)blk, (uint32_t)((unsigned long long)blk >> 32), (uint32_t)I.stream_id,
                   (uint32_t)(I.stream_id >> 32)};
  philox4x32_10(c, (uint32_t)I.seed, (uint32_t)(I.seed >> 32));
  float z[4];
  box_muller(c[0], c[1], z[0], z[1]);
  box_muller(c[2], c[3], z[2], z[3]);
  const int j = (int)(e0 % tab.d);   // d % 4 == 0: the four draws stay inside one sample
  const float4 m = *reinterpret_cast<const float4 *>(tab.mu + (size_t)(tab.item0 + it) * tab.d + j);
  const float4 v = *reinterpret_cast<const float4 *>(tab.var + (size_t)(tab.item0 + it) * tab.d + j);
  const float mm[4] = {m.x, m.y, m.z, m.w}, vv[4] = {v.x, v.y, v.z, v.w};
  T *dst = reinterpret_cast<T *>(tab.h_tilde) + (size_t)it * tab.S * tab.d + e0;
  T *dst2 = tab.h_tilde_out ? reinterpret_cast<T *>(tab.h_tilde_out) + (size_t)(tab.item0 + it) * tab.S * tab.d + e0
                            : nullptr;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const T hv = from_f32<T>(fmaf(sqrtf(vv[i]), z[i], mm[i]));
    dst[i] = hv;
    if (dst2) dst2[i] = hv;
  }
}

// ---- bf16 MFMA projection.  grid (ceil(n_out/256), ksplits, item groups), 512 threads (8 waves x 32 outputs).
// A group is a run of items with the same W_q; its n x S sampled states (contiguous in the workspace) are the
// columns of one product.
// WAVES: 8, or 16 for a single 32-column block (the staged columns are then shared by 512 outputs and a CU still
// holds sixteen waves when the 1024-channel slice leaves room for only one workgroup)
template <int NSB, int WAVES>
__global__ __launch_bounds__(WAVES * 64) void project_mfma_kernel(const SampleTable tab) {
  constexpr int kProjWaves = WAVES;
  extern __shared__ __align__(16) unsigned char smem[];
  bf16_t *Bs = reinterpret_cast<bf16_t *>(smem);   // [32*NSB][kslice + 8]
  const int it = tab.grp_first[blockIdx.z], ks = blockIdx.y;
  const int S_grp = tab.grp_count[blockIdx.z] * tab.S;     // columns of this product
  const int k0 = ks * tab.kslice;
  const int klen = min(tab.kslice, tab.d - k0);
  const int ldb = tab.kslice + 8;
  const bf16_t *hsrc = reinterpret_cast<const bf16_t *>(tab.h_tilde) + (size_t)it * tab.S * tab.d + k0;
  const int vec_per_row = tab.kslice / 8;
  auto stage_b = [&]() __attribute__((always_inline)) {
    for (int v = threadIdx.x; v < 32 * NSB * vec_per_row; v += kProjWaves * 64) {
      const int s = v / vec_per_row, kk = (v % vec_per_row) * 8;
      uint4 val = make_uint4(0, 0, 0, 0);
      if (s < S_grp && kk < klen) val = *reinterpret_cast<const uint4 *>(hsrc + (size_t)s * tab.d + kk);
      *reinterpret_cast<uint4 *>(Bs + s * ldb + kk) = val;
    }
    __syncthreads();
  };

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 31, hf = lane >> 5;
  floatx16 acc[NSB];
#pragma unroll
  for (int sb = 0; sb < NSB; ++sb)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[sb][r] = 0.f;

  // One k-step = 64 channels = 128 bytes of each of the wave's 32 W_q rows.  The rows are fetched with
  // fully coalesced non-temporal loads (8 lanes x 16 B cover a row's 128 bytes, a wave-wide load takes 8
  // rows), dropped into a wave-private XOR-swizzled LDS tile and read back in MFMA operand order: lane
  // (row, hf) takes channels hf*32 + i*8 .. +7 for MFMA i, the B operand uses the same assignment.  The
  // next k-step's loads are in flight while the current one is multiplied.  Rows beyond n_out re-read the
  // last row (their products are never stored); a shorter last k-slice takes the guarded path below.
  unsigned char *wtile = smem + (size_t)32 * NSB * ldb * sizeof(bf16_t) + wave * 4096;
  const int ob = blockIdx.x * (kProjWaves * 32) + wave * 32;
  const int lrow = lane >> 3, lpiece = lane & 7;
  const bf16_t *wbase = reinterpret_cast<const bf16_t *>(tab.it[it].w_q) + k0 + lpiece * 8;
  auto fetch_w = [&](u32x4_t(&w)[4], int kk) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int o = min(ob + 8 * j + lrow, tab.n_out - 1);
      w[j] = load_stream16(wbase + (size_t)o * tab.d + kk);
    }
  };
  auto stage_w = [&](const u32x4_t(&w)[4]) __attribute__((always_inline)) {
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int row = 8 * j + lrow;
      *reinterpret_cast<u32x4_t *>(wtile + row * 128 + ((lpiece ^ (row & 7)) << 4)) = w[j];
    }
  };
  auto mma = [&](int kk) __attribute__((always_inline)) {
    bf16x8 a[4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
      a[i] = *reinterpret_cast<const bf16x8 *>(wtile + col * 128 + (((hf * 4 + i) ^ (col & 7)) << 4));
#pragma unroll
    for (int sb = 0; sb < NSB; ++sb) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const uint4 raw = *reinterpret_cast<const uint4 *>(Bs + (sb * 32 + col) * ldb + kk + hf * 32 + i * 8);
        acc[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], __builtin_bit_cast(bf16x8, raw), acc[sb], 0, 0, 0);
      }
    }
  };
  if (klen == tab.kslice) {          // full slice: straight-line loads
    u32x4_t w0[4], w1[4];            // two k-steps in flight
    const int klast = tab.kslice - 64;
    fetch_w(w0, 0);                  // the first W_q rows are on their way while the sampled states are staged
    fetch_w(w1, min(64, klast));
    stage_b();
    for (int kk = 0; kk < tab.kslice; kk += 128) {
      stage_w(w0);
      fetch_w(w0, min(kk + 128, klast));             // (past the end a step is fetched again: no conditional load)
      __builtin_amdgcn_wave_barrier();
      mma(kk);
      __builtin_amdgcn_wave_barrier();
      if (kk + 64 < tab.kslice) {
        stage_w(w1);
        fetch_w(w1, min(kk + 192, klast));
        __builtin_amdgcn_wave_barrier();
        mma(kk + 64);
        __builtin_amdgcn_wave_barrier();
      }
    }
  } else {                           // the last, shorter slice: guarded element-wise loads
    stage_b();
    const int o = min(ob + col, tab.n_out - 1);
    const bf16_t *wrow = reinterpret_cast<const bf16_t *>(tab.it[it].w_q) + (size_t)o * tab.d + k0 + hf * 32;
    for (int kk = 0; kk < tab.kslice; kk += 64) {
      bf16x8 a[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint4 raw = make_uint4(0, 0, 0, 0);
        if (kk + hf * 32 + i * 8 < klen) raw = *reinterpret_cast<const uint4 *>(wrow + kk + i * 8);
        a[i] = __builtin_bit_cast(bf16x8, raw);
      }
#pragma unroll
      for (int sb = 0; sb < NSB; ++sb) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const uint4 raw = *reinterpret_cast<const uint4 *>(Bs + (sb * 32 + col) * ldb + kk + hf * 32 + i * 8);
          acc[sb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], __builtin_bit_cast(bf16x8, raw), acc[sb], 0, 0, 0);
        }
      }
    }
  }
  // C layout of the 32x32 MFMA: register r of lane l holds row 8*(r/4) + 4*(l/32) + r%4, column l%32.
  // Rows are outputs o, columns are samples.
#pragma unroll
  for (int sb = 0; sb < NSB; ++sb) {
    const int v = sb * 32 + col;           // column = (item of the group, sample)
    const int gi = v / tab.S, sm = v - gi * tab.S;
    float *part = tab.partial + ((size_t)((it + gi) * tab.ksplits + ks) * tab.n_out) * tab.SPs + sm;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int oo = ob + 8 * (r / 4) + 4 * hf + (r % 4);
      if (oo < tab.n_out && v < S_grp) part[(size_t)oo * tab.SPs] = acc[sb][r];
    }
  }
}

// ---- any storage type: one wave per output row, eight samples at a time.  grid (ceil(n_out/4), items)
template <typename T>
__global__ __launch_bounds__(256) void project_generic_kernel(const SampleTable tab) {
  constexpr int NV = Vec16<T>::N;
  const int it = blockIdx.y;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int o = blockIdx.x * 4 + wave;
  if (o >= tab.n_out) return;
  const T *wrow = reinterpret_cast<const T *>(tab.it[it].w_q) + (size_t)o * tab.d;
  const T *h = reinterpret_cast<const T *>(tab.h_tilde) + (size_t)it * tab.S * tab.d;
  float *part = tab.partial + ((size_t)it * tab.n_out + o) * tab.SPs;
  for (int s0 = 0; s0 < tab.SPs; s0 += 8) {
    typename Acc<T>::type acc[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc[u] = 0;
    for (int j = lane * NV; j < tab.d; j += 64 * NV) {
      float w[NV];
      Vec16<T>::load(wrow + j, w);
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        if (s0 + u < tab.S) {
          float x[NV];
          Vec16<T>::load(h + (size_t)(s0 + u) * tab.d + j, x);
#pragma unroll
          for (int i = 0; i < NV; ++i)
            acc[u] = fma((typename Acc<T>::type)w[i], (typename Acc<T>::type)x[i], acc[u]);
        }
      }
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      typename Acc<T>::type a = acc[u];
      for (int off = 32; off > 0; off >>= 1) a += __shfl_xor(a, off, 64);
      if (lane == 0) part[s0 + u] = (float)a;
    }
  }
}

// ---- reduction over k-splits, bias, rotation, rounding.  grid (query heads, items, blocks of 16 samples), 256
// threads: one workgroup per head and sample block: the partial sums are read along the samples (they are contiguous per output), the
// rotated pair goes into an LDS tile [sample][head_dim], and the tile is written out row by row, so that the stores
// to Q~ are contiguous runs of a head instead of two-byte stores n_out apart.
// kRopeSamples: 16, or 32 when there are more than 16 samples (a partial-sum row is then read whole by one workgroup)
template <typename T, int kRopeSamples>
__global__ __launch_bounds__(256) void rope_finalize_kernel(const SampleTable tab) {
  const int it = blockIdx.y, hd = blockIdx.x;
  const SampleItem I = tab.it[it];
  const int dk = tab.head_dim, half = dk / 2;          // head_dim <= 256 (checked by the entry point)
  __shared__ float cs[128][2];
  __shared__ T tile[kRopeSamples][256];
  for (int i = threadIdx.x; i < half; i += 256) {
    const double omega = pow((double)tab.theta, -2.0 * (double)i / (double)dk);
    double c = 0.0, s = 0.0;
    for (int tau = 0; tau < I.n_future; ++tau) {
      const double ang = (double)(I.pos0 + tau) * omega;
      c += cos(ang);
      s += sin(ang);
    }
    cs[i][0] = (float)(c / (double)I.n_future);
    cs[i][1] = (float)(s / (double)I.n_future);
  }
  __syncthreads();
  const T *bias = reinterpret_cast<const T *>(I.b_q);
  T *q = reinterpret_cast<T *>(tab.q_out) + (size_t)(tab.item0 + it) * tab.S * tab.n_out + (size_t)hd * dk;
  {
    const int s0 = blockIdx.z * kRopeSamples;
    for (int w = threadIdx.x; w < half * kRopeSamples; w += 256) {
      const int sl = w % kRopeSamples, i = w / kRopeSamples, s = s0 + sl;
      if (s < tab.S) {
        const int o1 = hd * dk + i, o2 = o1 + half;
        float a = 0.f, b = 0.f;
#pragma unroll 4
        for (int ks = 0; ks < tab.ksplits; ++ks) {
          const float *part = tab.partial + ((size_t)(it * tab.ksplits + ks) * tab.n_out) * tab.SPs;
          a += part[(size_t)o1 * tab.SPs + s];
          b += part[(size_t)o2 * tab.SPs + s];
        }
        if (bias) {
          a += to_f32<T>(bias[o1]);
          b += to_f32<T>(bias[o2]);
        }
        const float c = cs[i][0], sn = cs[i][1];
        tile[sl][i] = from_f32<T>(a * c - b * sn);
        tile[sl][i + half] = from_f32<T>(b * c + a * sn);
      }
    }
    __syncthreads();
    for (int e = threadIdx.x; e < kRopeSamples * dk; e += 256) {
      const int r = e / dk, c = e - r * dk;
      if (s0 + r < tab.S) q[(size_t)(s0 + r) * tab.n_out + c] = tile[r][c];
    }
  }
}

bool use_mfma(const gvote_shape *sh, int S) { return sh->dtype == GVOTE_BF16 && S <= 128; }

}  // namespace

SamplePlan plan_sample(const gvote_shape *sh, int n_items, int S) {
  SamplePlan p;
  p.SP = (S + 31) / 32 * 32;
  p.SPs = (S + 7) / 8 * 8;
  if (use_mfma(sh, S)) {
    // k-slices of 512 channels (a multiple of the 64-channel MFMA step); the last may be shorter.  With
    // 97..128 samples the staged sample block of a 512-channel slice (128 x 520 x 2 B) plus the wave tiles
    // would not fit the 160 KiB of LDS: those calls use 256-channel slices (100 KiB).
    const int full = p.SP > 96 ? 256 : 512;
    p.kslice = sh->d_model < full ? (sh->d_model + 63) / 64 * 64 : full;
    p.ksplits = (sh->d_model + p.kslice - 1) / p.kslice;
  } else {
    p.kslice = sh->d_model;
    p.ksplits = 1;
  }
  const int nb = n_items < kMaxItems ? n_items : kMaxItems;
  const size_t n_out = (size_t)sh->n_q_heads * sh->head_dim;
  p.h_bytes_per_item = align_up((size_t)S * sh->d_model * elem_bytes(sh->dtype), 256);
  p.partial_bytes_per_item = (size_t)p.ksplits * n_out * p.SPs * sizeof(float);
  p.ws_bytes = nb * (p.h_bytes_per_item + p.partial_bytes_per_item);
  return p;
}

gvote_status launch_sample(const gvote_shape *sh, const gvote_item *items, int n_items, int S, const float *mu,
                           const float *var, void *q_out, void *h_tilde_out, void *ws, hipStream_t st) {
  const SamplePlan plan = plan_sample(sh, n_items, S);
  const int n_out = sh->n_q_heads * sh->head_dim;
  const bool mfma = use_mfma(sh, S);
  for (int b0 = 0; b0 < n_items; b0 += kMaxItems) {
    const int nb = n_items - b0 < kMaxItems ? n_items - b0 : kMaxItems;
    SampleTable tab;
    tab.n_items = nb; tab.d = sh->d_model; tab.S = S; tab.SP = plan.SP; tab.SPs = plan.SPs; tab.pad1 = 0;
    tab.n_out = n_out; tab.head_dim = sh->head_dim; tab.ksplits = plan.ksplits; tab.kslice = plan.kslice;
    tab.theta = sh->rope_theta; tab.item0 = b0;
    tab.mu = mu; tab.var = var;
    tab.h_tilde = ws;
    tab.h_tilde_out = h_tilde_out;
    tab.partial = reinterpret_cast<float *>(reinterpret_cast<char *>(ws) +
                                            (size_t)(n_items < kMaxItems ? n_items : kMaxItems) * plan.h_bytes_per_item);
    tab.q_out = q_out;
    for (int i = 0; i < nb; ++i) {
      const gvote_item &g = items[b0 + i];
      SampleItem &s = tab.it[i];
      s.w_q = g.w_q; s.b_q = g.b_q; s.seed = g.seed; s.stream_id = g.stream_id;
      s.pos0 = g.pos0; s.n_future = g.n_future;
    }
    // the h~ rows of one item are S*d elements apart in the workspace (dense), see sample_hidden_kernel
    const dim3 gs(ceil_div((int64_t)S * sh->d_model / 4, 256), nb);
    if (sh->dtype == GVOTE_F32)
      hipLaunchKernelGGL(sample_hidden_kernel<float>, gs, dim3(256), 0, st, tab);
    else
      hipLaunchKernelGGL(sample_hidden_kernel<bf16_t>, gs, dim3(256), 0, st, tab);
    GVOTE_CHECK_LAUNCH();
    if (mfma) {
      // groups of consecutive items with one W_q; up to 96 columns per product (three 32-column MFMA blocks: the
      // staged columns of a 512-channel slice then still fit the LDS)
      const int per_group = S <= 96 ? 96 / S : 1;
      int widest = 0;
      tab.n_groups = 0;
      for (int i = 0; i < nb; ++i) {
        const int gl = tab.n_groups - 1;
        if (gl >= 0 && items[b0 + i].w_q == items[b0 + tab.grp_first[gl]].w_q && tab.grp_count[gl] < per_group) {
          ++tab.grp_count[gl];
        } else {
          tab.grp_first[tab.n_groups] = (unsigned char)i;
          tab.grp_count[tab.n_groups] = 1;
          ++tab.n_groups;
        }
        if (tab.grp_count[tab.n_groups - 1] > widest) widest = tab.grp_count[tab.n_groups - 1];
      }
      const int nsb = (widest * S + 31) / 32;
      // A product of up to 32 columns can take slices of 1024 channels (99 KB of LDS): half the partial sums for
      // rope_finalize to read, -8 % on the stage.  Only when 1024 divides the hidden size (a shorter last slice takes
      // the slow guarded path); the workspace is sized for the 512-channel slices either way.
      // Both only pay when the grid still fills the chip twice over (a single layer has few workgroups as it is).
      const long long wgs8 = (long long)ceil_div(n_out, 8 * 32) * tab.n_groups;      // per k-slice, 8-wave workgroups
      if (nsb == 1 && plan.kslice == 512 && sh->d_model % 1024 == 0 && wgs8 * (sh->d_model / 1024) >= 1024) {
        tab.kslice = 1024;
        tab.ksplits = sh->d_model / 1024;
      }
      const int waves = (nsb == 1 && tab.kslice == 1024 && wgs8 / 2 * tab.ksplits >= 512) ? 16 : 8;
      const dim3 gp(ceil_div(n_out, waves * 32), tab.ksplits, tab.n_groups);
      const size_t lds = (size_t)(32 * nsb) * (tab.kslice + 8) * sizeof(bf16_t) + waves * 4096;
      if (lds > kLdsBytesPerCu) return GVOTE_ERR_CAPACITY;       // cannot happen with the slices plan_sample picks
      hipError_t attr = hipSuccess;                               // more than 64 KiB of dynamic LDS must be asked for
      if (nsb == 1 && lds > 65536)
        attr = waves == 16 ? hipFuncSetAttribute(reinterpret_cast<const void *>(project_mfma_kernel<1, 16>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds)
                           : hipFuncSetAttribute(reinterpret_cast<const void *>(project_mfma_kernel<1, 8>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (nsb == 2 && lds > 65536)
        attr = hipFuncSetAttribute(reinterpret_cast<const void *>(project_mfma_kernel<2, 8>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (nsb == 3)
        attr = hipFuncSetAttribute(reinterpret_cast<const void *>(project_mfma_kernel<3, 8>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (nsb == 4)
        attr = hipFuncSetAttribute(reinterpret_cast<const void *>(project_mfma_kernel<4, 8>),
                                   hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
      if (attr != hipSuccess) return GVOTE_ERR_HIP;
      if (nsb == 1 && waves == 16)
        hipLaunchKernelGGL((project_mfma_kernel<1, 16>), gp, dim3(waves * 64), lds, st, tab);
      else if (nsb == 1)
        hipLaunchKernelGGL((project_mfma_kernel<1, 8>), gp, dim3(waves * 64), lds, st, tab);
      else if (nsb == 2)
        hipLaunchKernelGGL((project_mfma_kernel<2, 8>), gp, dim3(waves * 64), lds, st, tab);
      else if (nsb == 3)
        hipLaunchKernelGGL((project_mfma_kernel<3, 8>), gp, dim3(waves * 64), lds, st, tab);
      else
        hipLaunchKernelGGL((project_mfma_kernel<4, 8>), gp, dim3(waves * 64), lds, st, tab);
    } else {
      const dim3 gp(ceil_div(n_out, 4), nb);
      if (sh->dtype == GVOTE_F32)
        hipLaunchKernelGGL(project_generic_kernel<float>, gp, dim3(256), 0, st, tab);
      else
        hipLaunchKernelGGL(project_generic_kernel<bf16_t>, gp, dim3(256), 0, st, tab);
    }
    GVOTE_CHECK_LAUNCH();
    const int rope_block = S > 16 ? 32 : 16;
    const dim3 gf(n_out / sh->head_dim, nb, ceil_div(S, rope_block));
    if (sh->dtype == GVOTE_F32) {
      if (rope_block == 32) hipLaunchKernelGGL((rope_finalize_kernel<float, 32>), gf, dim3(256), 0, st, tab);
      else hipLaunchKernelGGL((rope_finalize_kernel<float, 16>), gf, dim3(256), 0, st, tab);
    } else {
      if (rope_block == 32) hipLaunchKernelGGL((rope_finalize_kernel<bf16_t, 32>), gf, dim3(256), 0, st, tab);
      else hipLaunchKernelGGL((rope_finalize_kernel<bf16_t, 16>), gf, dim3(256), 0, st, tab);
    }
    GVOTE_CHECK_LAUNCH();
  }
  return GVOTE_OK;
}

gvote_status launch_philox_u32(uint64_t seed, uint64_t stream_id, int64_t n, uint32_t *out, hipStream_t st) {
  if (n == 0) return GVOTE_OK;
  const int64_t blocks = (n + 3) / 4;
  hipLaunchKernelGGL(philox_u32_kernel, dim3((unsigned)((blocks + 255) / 256)), dim3(256), 0, st,
                     (unsigned long long)seed, (unsigned long long)stream_id, (long long)n, out);
  GVOTE_CHECK_LAUNCH();
  return GVOTE_OK;
}

}  // namespace gvote
