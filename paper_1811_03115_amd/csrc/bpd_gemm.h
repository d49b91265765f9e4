// Tuned bf16 MFMA GEMM kernels of libbpd (gfx950).  Included by bpd_kernels.h.
//
// Two regimes of the decoding step:
//   * "skinny": the M = B*k block rows fit one 16-row MFMA tile (batch-1 decoding).  The step
//     is then a chain of ~50 dependent small kernels whose cost is latency, not arithmetic:
//     every global load a wave will need is issued in one batch at kernel entry (weights
//     first, they do not depend on the previous kernel), LayerNorm is fused in as a prologue,
//     and K is split over the 4 waves of a workgroup so that a matrix with only N/16 column
//     tiles still spreads over N/16 CUs.
//   * "ldsx": many rows (batched decoding, the k*k-row vocabulary projection).  Weights go
//     straight from global memory into MFMA operand registers (the tiled layout makes each
//     16x32 tile one coalesced 1 KiB load, and no two waves of a workgroup share a weight
//     tile), activations are staged through LDS where all 4 waves reuse them.
#pragma once

// With e.stats_out (mode 0): per 16-column tile and row the sum and the sum of squares of the stored values go to
// stats_out[(tile * M + row) * 2 + {0, 1}], for the LayerNorm that the next GEMM applies while it stages its activations.
// ROWAFF: the products are finished as rstd * (acc - mu * c[n]) + d[n] first (LayerNorm folded into the weights, see
// Epi); ms: (mu, rstd) of the workgroup's rows, in LDS.
// pre_b / pre_r (with e.pre_epi): bias of the NT column tiles and residual of the MT x NT tiles, fetched at kernel entry.
template <int MT, int NT, bool STATS, bool ROWAFF = false>
__device__ __forceinline__ void store_tiles(const Epi& e_in, int g, const f32x4 (&acc)[MT][NT], int m0, int nt0,
                                            int ntiles, int M, int lane, const float2* ms = nullptr,
                                            const float4* rc = nullptr, const float4* rd = nullptr,
                                            const float4* pre_b = nullptr, const float4* pre_r = nullptr,
                                            unsigned char* stage = nullptr) {
  const bool stats = STATS && e_in.mode == 0 && e_in.stats_out != nullptr;
  // bf16 output of four whole column tiles per wave (64 columns: 128 bytes per row), `stage`: 2 KB of LDS of this wave's
  // own.  Stored straight from the accumulator layout a lane holds 4 columns (8 bytes) of a row and a store instruction
  // touches 16 rows x 32 bytes; the 27 MB that the heads' hidden layers write at batch 32 went out at 1.4 TB/s that way
  // (6.7 of the kernel's 33 us with one row block).  Instead the row tile's 16 x 64 values pass through LDS (16-byte
  // segments XOR-ed with the row, conflict-free both ways) and leave as 16 bytes per lane: 8 rows x 128 bytes per store.
  const bool wide = NT == 4 && stage != nullptr && e_in.mode == 0 && e_in.Ya != nullptr && nt0 + NT <= ntiles &&
                    (e_in.ldya & 7) == 0 && (e_in.ya_g & 7) == 0 && ((size_t)e_in.Ya & 15) == 0;
  bf16_t* ya = (bf16_t*)e_in.Ya;
  Epi e = e_in;
  if (wide) e.Ya = nullptr;                      // the per-tile stores below then skip the bf16 output
  float2 wsum[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) wsum[t] = make_float2(0.f, 0.f);
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int m = m0 + t * 16 + (lane & 15);
    float2 mr = make_float2(0.f, 1.f);
    if constexpr (ROWAFF) mr = ms[t * 16 + (lane & 15)];
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      if (nt0 + u >= ntiles) continue;            // the same for the whole wave
      const int n = (nt0 + u) * 16 + (lane >> 4) * 4;
      float v[4] = {acc[t][u][0], acc[t][u][1], acc[t][u][2], acc[t][u][3]};
      if constexpr (ROWAFF) {
        const float4 cc = rc[u], dd = rd[u];     // fetched at kernel entry: no round trip here
        v[0] = mr.y * (v[0] - mr.x * cc.x) + dd.x; v[1] = mr.y * (v[1] - mr.x * cc.y) + dd.y;
        v[2] = mr.y * (v[2] - mr.x * cc.z) + dd.z; v[3] = mr.y * (v[3] - mr.x * cc.w) + dd.w;
      }
      float fin[4] = {0.f, 0.f, 0.f, 0.f};
      if (pre_b != nullptr && e.pre_epi) {       // mode 0 with its operands at hand (pre_b is a compile-time null elsewhere)
        const float4 bs = pre_b[u], rv = pre_r[t * NT + u];
        v[0] += bs.x; v[1] += bs.y; v[2] += bs.z; v[3] += bs.w;
        if (e.relu) { v[0] = fmaxf(v[0], 0.f); v[1] = fmaxf(v[1], 0.f); v[2] = fmaxf(v[2], 0.f); v[3] = fmaxf(v[3], 0.f); }
        v[0] += rv.x; v[1] += rv.y; v[2] += rv.z; v[3] += rv.w;
        if (m < M) {
          if (e.Yf) *(float4*)(e.Yf + g * e.yf_g + (long)m * e.ldyf + n) = make_float4(v[0], v[1], v[2], v[3]);
          if (e.Ya) *(uint2*)((bf16_t*)e.Ya + g * e.ya_g + (long)m * e.ldya + n) =
                        make_uint2((unsigned)f2bf(v[0]) | ((unsigned)f2bf(v[1]) << 16), (unsigned)f2bf(v[2]) | ((unsigned)f2bf(v[3]) << 16));
          fin[0] = v[0]; fin[1] = v[1]; fin[2] = v[2]; fin[3] = v[3];
        }
      } else if (m < M) epi_store4f(e, g, m, n, v, fin);
      if (wide) {                                 // (the direct stores above saw e.Ya == nullptr: see the copy of e below)
        const int lr_ = lane & 15, sg = (u * 2 + (lane >> 5)) ^ (lr_ & 7);
        *(uint2*)(stage + lr_ * 128 + sg * 16 + ((lane >> 4) & 1) * 8) =
            make_uint2((unsigned)f2bf(fin[0]) | ((unsigned)f2bf(fin[1]) << 16), (unsigned)f2bf(fin[2]) | ((unsigned)f2bf(fin[3]) << 16));
      }
      if (stats) {
        float sv = (fin[0] + fin[1]) + (fin[2] + fin[3]);
        float qv = (fin[0] * fin[0] + fin[1] * fin[1]) + (fin[2] * fin[2] + fin[3] * fin[3]);
        sv += __shfl_xor(sv, 16, 64); sv += __shfl_xor(sv, 32, 64);
        qv += __shfl_xor(qv, 16, 64); qv += __shfl_xor(qv, 32, 64);
        wsum[t].x += sv; wsum[t].y += qv;        // this wave's NT tiles lie in one 64-column block
      }
    }
    if (wide) {
#pragma unroll
      for (int h = 0; h < 2; ++h) {
        const int r = h * 8 + (lane >> 3), sgr = lane & 7;
        const uint4 w = *(const uint4*)(stage + r * 128 + ((sgr ^ (r & 7)) * 16));
        const int mm = m0 + t * 16 + r;
        if (mm < M) *(uint4*)(ya + g * e.ya_g + (long)mm * e.ldya + nt0 * 16 + sgr * 8) = w;
      }
    }
  }
  if constexpr (STATS) {
    // statistics per 64-column block and row: the waves that share a block (4 / NT of them) meet in LDS; the host
    // launches this variant only when N is a multiple of 64 * NT, so every wave of the workgroup gets here
    if (stats) {
      static_assert(NT == 1 || NT == 2 || NT == 4, "a wave's tiles stay inside one 64-column block");
      __shared__ float2 st_x[4][16 * MT];
      const int wave = threadIdx.x >> 6;
#pragma unroll
      for (int t = 0; t < MT; ++t)
        if (lane < 16) st_x[wave][t * 16 + lane] = wsum[t];
      __syncthreads();
      constexpr int G = 4 / NT, BMs = 16 * MT;
      const int blk0 = (nt0 - wave * NT) >> 2;   // first 64-column block of the workgroup
      for (int idx = threadIdx.x; idx < NT * BMs; idx += 256) {
        const int j = idx / BMs, r = idx - j * BMs;
        float2 a = st_x[j * G][r];
#pragma unroll
        for (int w = 1; w < G; ++w) { a.x += st_x[j * G + w][r].x; a.y += st_x[j * G + w][r].y; }
        if (m0 + r < M) ((float2*)e.stats_out)[(long)(blk0 + j) * M + m0 + r] = a;
      }
    }
  }
}

// Row-wise arg-max over this wave's columns, merged into keys[] with a 64-bit atomic max.
template <int MT, int NT>
__device__ __forceinline__ void argmax_tiles(const f32x4 (&acc)[MT][NT], int m0, int nt0, int ntiles, int M, int N,
                                             int lane, unsigned long long* keys, float* logits) {
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int m = m0 + t * 16 + (lane & 15);
    unsigned long long best = 0ull;
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      if (nt0 + u >= ntiles) continue;
      const int n = (nt0 + u) * 16 + (lane >> 4) * 4;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float v = acc[t][u][r];
        const unsigned long long key = argmax_key(v, (unsigned)(n + r));
        best = key > best ? key : best;
        if (logits && m < M) logits[(long)m * N + n + r] = v;
      }
    }
    unsigned long long o = __shfl_xor(best, 16, 64); best = o > best ? o : best;
    o = __shfl_xor(best, 32, 64); best = o > best ? o : best;
    if (lane < 16 && m < M) atomicMax(&keys[m], best);
  }
}

// ---------------------------------------------------------------------------------------
// LayerNorm statistics travel with the residual stream: every kernel that writes x (16-column
// tile by tile) also writes, per tile and row, the partial sum and sum of squares of its 16
// new values; a consumer adds the d/16 partials of a row in a fixed order.  This removes the
// LayerNorm kernels and any cross-lane reduction over a whole row from the latency chain.
//   stats[(tile * 16 + row) * 2 + {0,1}],  tile < K/16 <= 64, row < 16.
__device__ __forceinline__ void row_stats_load(const float* stats, int K, int lane, float2 (&v)[16]) {
  const int m = lane & 15, part = lane >> 4, slots = K >> 4;
  // branch-free on purpose: conditional loads make the compiler wait for each one in turn
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const int t = part + 4 * i;
    v[i] = ((const float2*)stats)[(t < slots ? t : 0) * 16 + m];
  }
}
__device__ __forceinline__ void row_stats_reduce(const float2 (&v)[16], int K, float eps, int lane, float& mu, float& rstd) {
  const int part = lane >> 4, slots = K >> 4;
  float s = 0.f, q = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) {
    const float w = (part + 4 * i) < slots ? 1.f : 0.f;
    s = fmaf(w, v[i].x, s); q = fmaf(w, v[i].y, q);
  }
  s += __shfl_xor(s, 16, 64); s += __shfl_xor(s, 32, 64);
  q += __shfl_xor(q, 16, 64); q += __shfl_xor(q, 32, 64);
  mu = s / K;
  const float var = fmaxf(q / K - mu * mu, 0.f);
  rstd = 1.0f / sqrtf(var + eps);
}
__device__ __forceinline__ void row_stats(const float* stats, int K, float eps, int lane, float& mu, float& rstd) {
  float2 v[16];
  row_stats_load(stats, K, lane, v);
  __builtin_amdgcn_sched_barrier(0);
  row_stats_reduce(v, K, eps, lane, mu, rstd);
}

struct LnP {
  const float* x;       // [M][K] fp32 residual stream (row stride K)
  const float* g;       // [K]
  const float* b;       // [K]
  const float* stats;   // partial sums written by the producer of x
  float eps;
};

__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) { return (unsigned)f2bf(lo) | ((unsigned)f2bf(hi) << 16); }

// Skinny GEMM: blocks of 16*MT rows (blockIdx.y), all rows of a block resident in registers.  Workgroup = WAVES waves
// sharing NT column tiles, K split WAVES ways (wave w takes k-steps w, w+WAVES, ...; at most U
// per wave, so K <= 32*WAVES*U).  A wave keeps its MT x U activation fragments in registers and
// streams weight tiles; per column-tile group the WAVES partial sums meet in LDS (double
// buffered: one barrier per group) and the MT*NT output tiles are finished by the waves in
// turn (tile id % WAVES).  A workgroup walks tile groups blockIdx.x, blockIdx.x + gridDim.x,
// ... with the weights of the next DEPTH groups in flight (DEPTH == 0: one group per
// workgroup).
//   XLN = false: X is bf16 [M][K] in global memory.
//   XLN = true : (MT == 1) X = LayerNorm(x) of the fp32 residual stream, normalised in
//                registers from the producer's partial statistics.
// Every global load of the first group (weights, activations, statistics, bias and residual of
// the epilogue) is issued before anything is waited for: one memory round trip per kernel.
// Epilogue (mode 0) additionally supports: R = LayerNorm(R) via e.lnR_* (the heads' residual
// is the normalised decoder output), and writing partial LayerNorm statistics of the result.
// Dynamic LDS: 2 * WAVES * MT * NT * 1024 bytes.
typedef unsigned int u32x4_nt __attribute__((ext_vector_type(4)));
// STREAM: the weight tiles are fetched with non-temporal loads.  A weight matrix that is read once
// per step and does not fit the last-level cache together with the rest of the model (the heads of
// Transformer-big) would otherwise evict the decoder layers' weights from it every step.
template <int MT, int NT, bool XLN, bool ARGMAX, int WAVES, int U, int DEPTH, bool STREAM>
__global__ __launch_bounds__(WAVES * 64) void skinny_gemm_kernel(GemmP p, Epi e, LnP ln, unsigned long long* keys,
                                                                  float* logits) {
  constexpr int TILES = MT * NT, OWN = (TILES + WAVES - 1) / WAVES;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  f32x4* red = (f32x4*)smem_raw;               // [2][WAVES][TILES][64]
  // XLN: LayerNorm gain and bias (K <= 1024 floats each) reach the lanes through LDS: one 16-byte
  // global load per thread instead of sixteen per lane (the address unit is the busy one here)
  constexpr int GBL = (2 * 1024 / 4 + WAVES * 64 - 1) / (WAVES * 64);      // float4 loads per thread
  __shared__ __attribute__((aligned(16))) float gb_s[XLN ? 2 * 1024 : 4];
  // partial LayerNorm statistics of the residual stream (XLN: of the input; otherwise of the epilogue's LayerNorm-ed
  // residual operand, if any), same layout as in global memory
  __shared__ __attribute__((aligned(16))) float st_s[(XLN || !ARGMAX) ? 64 * 16 * 2 : 4];
  static_assert(GBL <= 2, "gain/bias staging");
  float4 gb0 = make_float4(0.f, 0.f, 0.f, 0.f), gb1 = gb0;   // (named scalars: an indexed array would live in scratch)
  if (XLN) {
    const int nv = p.K >> 2;                   // float4 per vector; thread index 0 .. 2*nv-1: gain then bias
    const int i0 = threadIdx.x, i1 = threadIdx.x + WAVES * 64;
    gb0 = ((const float4*)(i0 < nv ? ln.g : ln.b))[i0 < nv ? i0 : (i0 < 2 * nv ? i0 - nv : 0)];
    if (GBL > 1) gb1 = ((const float4*)(i1 < nv ? ln.g : ln.b))[i1 < nv ? i1 : (i1 < 2 * nv ? i1 - nv : 0)];
  }
  float4 st0 = make_float4(0.f, 0.f, 0.f, 0.f), st1 = st0;   // statistics: (K/16) * 8 float4 in all
  const bool epi_ln = !XLN && !ARGMAX && e.mode == 0 && e.lnR_stats != nullptr;
  if (XLN || epi_ln) {
    const float* sp_ = XLN ? ln.stats : e.lnR_stats;
    const int ns4 = ((XLN ? p.K : e.lnR_K) >> 4) * 8;
    const int i0 = threadIdx.x, i1 = threadIdx.x + WAVES * 64;
    st0 = ((const float4*)sp_)[i0 < ns4 ? i0 : 0];
    if (GBL > 1) st1 = ((const float4*)sp_)[i1 < ns4 ? i1 : 0];
  }
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int g = blockIdx.z;
  const int ntiles = p.N >> 4, ksteps = p.K >> 5;
  const int lr = lane & 15, lk = (lane >> 4) * 8;
  const uint4* W = (const uint4*)((const bf16_t*)p.W + g * p.w_g) + lane;
  const uint4 zero4 = make_uint4(0, 0, 0, 0);
  int nt0 = blockIdx.x * NT;
  if (nt0 >= ntiles) return;
  const int mb0 = blockIdx.y * (16 * MT);       // row block of this workgroup

  constexpr bool PERSIST = DEPTH > 0;
  const int stride = gridDim.x * NT;            // distance between consecutive tile groups of this workgroup
  uint4 a[DEPTH + 1][U][NT];                    // a[0]: current group, a[1..DEPTH]: groups in flight
#define BPD_LOAD_A(dst, tile0)                                                              \
  _Pragma("unroll") for (int i = 0; i < U; ++i) {                                           \
    const int ks_ = wave + WAVES * i;                                                       \
    const int ksc_ = ks_ < ksteps ? ks_ : ksteps - 1;                                       \
    _Pragma("unroll") for (int u = 0; u < NT; ++u) {                                        \
      int t_ = (tile0) + u; t_ = t_ < ntiles ? t_ : ntiles - 1;                             \
      if (STREAM) dst[i][u] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_nt*)&W[((long)t_ * ksteps + ksc_) * 64])); \
      else dst[i][u] = W[((long)t_ * ksteps + ksc_) * 64];                                  \
    }                                                                                       \
  }
  BPD_LOAD_A(a[0], nt0)                         // weights first: they do not depend on the producer kernel
#pragma unroll
  for (int dd = 1; dd < DEPTH; ++dd)
    if (nt0 + dd * stride < ntiles) { BPD_LOAD_A(a[dd], nt0 + dd * stride) }

  // operands of the epilogue (bias, residual) for the tiles this wave will finish; the host passes
  // a zero-filled buffer where there is no bias / residual so that the loads are unconditional
  const bool plain_epi = !ARGMAX && e.mode == 0;
  float4 r_cur[OWN], bias_cur[OWN], r_nxt[OWN], bias_nxt[OWN];
#define BPD_LOAD_EPI(rdst, bdst, tile0)                                                     \
  if (!ARGMAX) {                                                                            \
    _Pragma("unroll") for (int j = 0; j < OWN; ++j) {                                       \
      int id_ = wave + WAVES * j; id_ = id_ < TILES ? id_ : TILES - 1;                      \
      const int t_ = id_ / NT, u_ = id_ % NT;                                               \
      int nt_ = (tile0) + u_; nt_ = nt_ < ntiles ? nt_ : ntiles - 1;                        \
      const int n_ = nt_ * 16 + (lane >> 4) * 4;                                            \
      int m_ = mb0 + t_ * 16 + lr; m_ = m_ < p.M ? m_ : p.M - 1;                                \
      rdst[j] = *(const float4*)(e.R + g * e.r_g + (long)m_ * e.ldr + n_);                  \
      bdst[j] = *(const float4*)(e.bias + g * e.bias_g + n_);                               \
    }                                                                                       \
  }
  BPD_LOAD_EPI(r_cur, bias_cur, nt0)
  __builtin_amdgcn_sched_barrier(0);            // keep the issue order: the scheduler would sink loads to their uses

  // activation fragments, kept for all tile groups of this workgroup
  uint4 b[MT][U];
  if (XLN) {
    const int mrow = mb0 + lr < p.M ? mb0 + lr : p.M - 1;
    float4 xv[U][2], gv[U][2], bv[U][2];
#pragma unroll
    for (int i = 0; i < U; ++i) {
      const int ks = wave + WAVES * i;
      const int col = (ks < ksteps ? ks : 0) * 32 + lk;
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) xv[i][hh] = *(const float4*)(ln.x + (long)mrow * p.K + col + 4 * hh);
    }
    __builtin_amdgcn_sched_barrier(0);
    {                                          // gain / bias were requested first, so they arrive first
      const int nv = p.K >> 2;
      const int i0 = threadIdx.x, i1 = threadIdx.x + WAVES * 64;
      if (i0 < 2 * nv) *(float4*)&gb_s[i0 < nv ? 4 * i0 : 1024 + 4 * (i0 - nv)] = gb0;
      if (GBL > 1 && i1 < 2 * nv) *(float4*)&gb_s[i1 < nv ? 4 * i1 : 1024 + 4 * (i1 - nv)] = gb1;
      const int ns4 = (p.K >> 4) * 8;
      if (i0 < ns4) *(float4*)&st_s[4 * i0] = st0;
      if (GBL > 1 && i1 < ns4) *(float4*)&st_s[4 * i1] = st1;
    }
    __syncthreads();
    float2 sv[16];
    row_stats_load(st_s, p.K, lane, sv);       // from LDS now
    float mu, rstd;
    row_stats_reduce(sv, p.K, ln.eps, lane, mu, rstd);
#pragma unroll
    for (int i = 0; i < U; ++i) {
      const int ks = wave + WAVES * i;
      const int col = (ks < ksteps ? ks : 0) * 32 + lk;
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        gv[i][hh] = *(const float4*)&gb_s[col + 4 * hh];
        bv[i][hh] = *(const float4*)&gb_s[1024 + col + 4 * hh];
      }
    }
#pragma unroll
    for (int i = 0; i < U; ++i) {
      float y[8];
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        y[4 * hh + 0] = (xv[i][hh].x - mu) * rstd * gv[i][hh].x + bv[i][hh].x;
        y[4 * hh + 1] = (xv[i][hh].y - mu) * rstd * gv[i][hh].y + bv[i][hh].y;
        y[4 * hh + 2] = (xv[i][hh].z - mu) * rstd * gv[i][hh].z + bv[i][hh].z;
        y[4 * hh + 3] = (xv[i][hh].w - mu) * rstd * gv[i][hh].w + bv[i][hh].w;
      }
      const uint4 yb = make_uint4(pack_bf16(y[0], y[1]), pack_bf16(y[2], y[3]), pack_bf16(y[4], y[5]), pack_bf16(y[6], y[7]));
      b[0][i] = (wave + WAVES * i) < ksteps ? yb : zero4;
    }
  } else {
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      int row = mb0 + t * 16 + lr; row = row < p.M ? row : p.M - 1;
      const bf16_t* xg = (const bf16_t*)p.X + g * p.x_g + (long)row * p.ldx + lk;
#pragma unroll
      for (int i = 0; i < U; ++i) {
        const int ks = wave + WAVES * i;
        const uint4 v = *(const uint4*)(xg + (ks < ksteps ? ks : ksteps - 1) * 32);
        b[t][i] = ks < ksteps ? v : zero4;          // k-steps beyond K contribute nothing
      }
    }
    __builtin_amdgcn_sched_barrier(0);
    if (epi_ln) {                              // read back after the barrier that follows the first group's MFMAs
      const int ns4 = (e.lnR_K >> 4) * 8;
      const int i0 = threadIdx.x, i1 = threadIdx.x + WAVES * 64;
      if (i0 < ns4) *(float4*)&st_s[4 * i0] = st0;
      if (GBL > 1 && i1 < ns4) *(float4*)&st_s[4 * i1] = st1;
    }
  }

  unsigned long long best_run[OWN];
#pragma unroll
  for (int j = 0; j < OWN; ++j) best_run[j] = 0ull;
  int it = 0;
  for (; nt0 < ntiles; nt0 += (PERSIST ? stride : ntiles), ++it) {
    f32x4 acc[MT][NT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int u = 0; u < NT; ++u) acc[t][u] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int nt_next = nt0 + stride;
    const bool more = PERSIST && nt_next < ntiles;
    if (PERSIST && nt0 + DEPTH * stride < ntiles) { BPD_LOAD_A(a[DEPTH], nt0 + DEPTH * stride) }
    if (more) { BPD_LOAD_EPI(r_nxt, bias_nxt, nt_next) }
#pragma unroll
    for (int i = 0; i < U; ++i)
#pragma unroll
      for (int t = 0; t < MT; ++t)
#pragma unroll
        for (int u = 0; u < NT; ++u)
          acc[t][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[0][i][u]),
                                                              __builtin_bit_cast(bf16x8, b[t][i]), acc[t][u], 0, 0, 0);
    // partial sums of all waves meet in LDS
    f32x4* rb = red + (it & 1) * (WAVES * TILES * 64);
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int u = 0; u < NT; ++u) rb[(wave * TILES + t * NT + u) * 64 + lane] = acc[t][u];
    __syncthreads();
    float mu = 0.f, rstd = 1.f;
    if (plain_epi && e.lnR_stats && wave < TILES) {
      if (XLN) row_stats(e.lnR_stats, e.lnR_K, e.lnR_eps, lane, mu, rstd);
      else row_stats(st_s, e.lnR_K, e.lnR_eps, lane, mu, rstd);
    }
#pragma unroll
    for (int j = 0; j < OWN; ++j) {
      const int id = wave + WAVES * j;
      if (id >= TILES) continue;
      const int t = id / NT, u = id % NT;
      if (nt0 + u >= ntiles) continue;
      f32x4 sum = rb[id * 64 + lane];
#pragma unroll
      for (int w = 1; w < WAVES; ++w) sum += rb[(w * TILES + id) * 64 + lane];
      const int m = mb0 + t * 16 + lr;
      const int n = (nt0 + u) * 16 + (lane >> 4) * 4;
      if (ARGMAX) {
        // running best over all column tiles this workgroup walks; merged into keys[] once at the end
        // (atomics on one row's key serialise, so their number is what matters)
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const unsigned long long key = argmax_key(sum[r], (unsigned)(n + r));
          best_run[j] = key > best_run[j] ? key : best_run[j];
        }
        if (logits && m < p.M) *(float4*)(logits + (long)m * p.N + n) = make_float4(sum[0], sum[1], sum[2], sum[3]);
      } else if (e.mode != 0) {
        if (m < p.M) {
          const float v4[4] = {sum[0], sum[1], sum[2], sum[3]};
          epi_store4(e, g, m, n, v4);
        }
      } else {
        float4 rv = r_cur[j];
        const float4 bs = bias_cur[j];
        if (e.lnR_stats) {
          const float4 gg = *(const float4*)(e.lnR_g + n), bb = *(const float4*)(e.lnR_b + n);
          rv.x = (rv.x - mu) * rstd * gg.x + bb.x; rv.y = (rv.y - mu) * rstd * gg.y + bb.y;
          rv.z = (rv.z - mu) * rstd * gg.z + bb.z; rv.w = (rv.w - mu) * rstd * gg.w + bb.w;
        }
        float v[4] = {sum[0] + bs.x, sum[1] + bs.y, sum[2] + bs.z, sum[3] + bs.w};
        if (e.relu) {
#pragma unroll
          for (int r = 0; r < 4; ++r) v[r] = fmaxf(v[r], 0.f);
        }
        v[0] += rv.x; v[1] += rv.y; v[2] += rv.z; v[3] += rv.w;
        if (e.stats_out) {          // MT == 1 on this path: row = lane % 16
          float sv = (v[0] + v[1]) + (v[2] + v[3]);
          float qv = (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
          sv += __shfl_xor(sv, 16, 64); sv += __shfl_xor(sv, 32, 64);
          qv += __shfl_xor(qv, 16, 64); qv += __shfl_xor(qv, 32, 64);
          if (lane < 16) ((float2*)e.stats_out)[(nt0 + u) * 16 + lane] = make_float2(sv, qv);
        }
        if (m < p.M) {
          if (e.Yf) *(float4*)(e.Yf + g * e.yf_g + (long)m * e.ldyf + n) = make_float4(v[0], v[1], v[2], v[3]);
          if (e.Ya) *(uint2*)((bf16_t*)e.Ya + g * e.ya_g + (long)m * e.ldya + n) =
                        make_uint2(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]));
        }
      }
    }
    if (more) {
#pragma unroll
      for (int dd = 0; dd < DEPTH; ++dd)
#pragma unroll
        for (int i = 0; i < U; ++i)
#pragma unroll
          for (int u = 0; u < NT; ++u) a[dd][i][u] = a[dd + 1][i][u];
#pragma unroll
      for (int j = 0; j < OWN; ++j) { r_cur[j] = r_nxt[j]; bias_cur[j] = bias_nxt[j]; }
    }
  }
  if (ARGMAX) {
#pragma unroll
    for (int j = 0; j < OWN; ++j) {
      const int id = wave + WAVES * j;
      if (id >= TILES) continue;
      const int m = mb0 + (id / NT) * 16 + lr;
      unsigned long long best = best_run[j];
      unsigned long long o = __shfl_xor(best, 16, 64); best = o > best ? o : best;
      o = __shfl_xor(best, 32, 64); best = o > best ? o : best;
      if (keys && lane < 16 && m < p.M && best != 0ull) atomicMax(&keys[m], best);
    }
  }
#undef BPD_LOAD_A
#undef BPD_LOAD_EPI
}

// ---------------------------------------------------------------------------------------
// Streaming skinny GEMM for a long-K weight stream that gives every CU several column tiles (the
// heads' output layers at batch 1: 640 tiles of 4096 x 16).  One 16-row block, K == 256 * U, mode-0
// epilogue without statistics output.  Grid (GX, 1, groups), 512 threads, one workgroup per CU.
// A workgroup owns the contiguous column tiles [t0, t1) of its group (at most 8):
//   * X (M rows x K, bf16) goes global -> LDS once (direct loads, rows padded by 16 bytes so that the
//     MFMA operand reads of a wave spread over all banks); the skinny kernel re-reads X per tile
//   * K is split over the 8 waves as in the skinny kernel (wave w takes k-steps w, w+8, ...: the same
//     summation order, so both kernels give the same bits); the 16 weight loads of the next tile are
//     issued before the current tile is multiplied, and the previous tile is finished (partials of
//     the 8 waves added by one wave, in turn) after that, so a wave always has 16-32 KiB in flight
//   * bias, residual rows and the LayerNorm vectors of the epilogue for all owned columns are
//     fetched once (one 16-byte load per thread) and read from LDS when a tile is finished
// Dynamic LDS: 16 KiB (partials, double buffered; the LayerNorm statistics pass through the
// second half before it is first used) + 8 KiB (residual rows) + 1.5 KiB (vectors) + M*(K+8)*2.
template <int U, bool STREAM>
__global__ __launch_bounds__(512) void stream_gemm_kernel(GemmP p, Epi e) {
  constexpr int WAVES = 8, TW = 8, EC = 16 * TW;      // EC: columns a workgroup may own
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  f32x4* red = (f32x4*)smem_raw;              // [2][WAVES][64]
  float* st_s = (float*)(smem_raw + 8192);    // [64][16][2], dead before red[1] is first written
  float* r_s = (float*)(smem_raw + 16384);    // [16][EC]
  float* v_s = r_s + 16 * EC;                 // [3][EC]
  bf16_t* xs = (bf16_t*)(v_s + 3 * EC);
  const int ldxs = p.K + 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane & 15, lq = lane >> 4;
  const int g = blockIdx.z;
  const int ntiles = p.N >> 4, ksteps = p.K >> 5;
  const int t0 = (int)(blockIdx.x * (unsigned)ntiles / gridDim.x), t1 = (int)((blockIdx.x + 1) * (unsigned)ntiles / gridDim.x);
  if (t0 >= t1) return;
  {   // X: global -> LDS directly, whole wave-loads of 64 pieces inside one row
    const int segs = p.K >> 3;                 // 16-byte pieces per row
    const bf16_t* xg = (const bf16_t*)p.X + g * p.x_g;
#pragma unroll
    for (int i = 0; i < U; ++i) {
      const int q0 = i * 512 + wave * 64;
      const int row = (unsigned)q0 / (unsigned)segs, seg0 = q0 - row * segs;
      if (row < p.M)
        __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(xg + (long)row * p.ldx + (seg0 + lane) * 8),
                                         (void __attribute__((address_space(3)))*)(xs + row * ldxs + seg0 * 8), 16, 0, 0);
    }
  }
  const bool has_ln = e.lnR_stats != nullptr;
  // small operands: statistics of the epilogue's LayerNorm, residual rows and the per-column vectors of this workgroup's columns
  float4 st0, st1, rr, vv;
  {
    const float* sp_ = has_ln ? e.lnR_stats : e.bias;
    const int ns4 = has_ln ? (e.lnR_K >> 4) * 8 : 1;
    st0 = ((const float4*)sp_)[tid < ns4 ? tid : 0];
    st1 = ((const float4*)sp_)[tid + 512 < ns4 ? tid + 512 : 0];
    const int nc4 = (t1 - t0) * 4;             // float4 per row of this workgroup's columns
    const int row = tid >> 5, c4 = tid & 31;
    const int c4c = c4 < nc4 ? c4 : 0;
    rr = *(const float4*)(e.R + g * e.r_g + (long)(row < p.M ? row : p.M - 1) * e.ldr + t0 * 16 + c4c * 4);
    const float* vp_ = row == 1 && has_ln ? e.lnR_g : (row == 2 && has_ln ? e.lnR_b : e.bias + g * e.bias_g);
    vv = *(const float4*)(vp_ + t0 * 16 + c4c * 4);
  }
  __builtin_amdgcn_sched_barrier(0);
  const char* Wg = (const char*)((const bf16_t*)p.W + g * p.w_g);      // wave-uniform; the lane adds 16 * lane
  const unsigned loff = lane * 16;
  uint4 a_cur[U], a_nxt[U];
#define ST_LOADW(dst, tile)                                                                     \
  _Pragma("unroll") for (int i = 0; i < U; ++i) {                                               \
    const char* wp_ = Wg + ((long)(tile) * ksteps + wave + WAVES * i) * 1024;                   \
    if (STREAM) dst[i] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_nt*)(wp_ + loff))); \
    else dst[i] = *(const uint4*)(wp_ + loff);                                                  \
  }
#define ST_SMALL_TO_LDS()                                                                       \
  {                                                                                             \
    const int ns4 = has_ln ? (e.lnR_K >> 4) * 8 : 0;                                            \
    if (tid < ns4) *(float4*)&st_s[4 * tid] = st0;                                              \
    if (tid + 512 < ns4) *(float4*)&st_s[4 * (tid + 512)] = st1;                                \
    *(float4*)&r_s[(tid >> 5) * EC + (tid & 31) * 4] = rr;                                      \
    if (tid < 96) *(float4*)&v_s[(tid >> 5) * EC + (tid & 31) * 4] = vv;                        \
  }
  const bf16_t* xrow = xs + (lr < p.M ? lr : p.M - 1) * ldxs + lq * 8;
  float mu = 0.f, rstd = 1.f;
  int it = 0;
#define ST_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))
#define ST_FINISH(tile, itv)                                                                    \
  if (wave == ((itv) & 7)) {                                                                    \
    const f32x4* rb_ = red + ((itv) & 1) * (WAVES * 64);                                        \
    f32x4 sum = rb_[lane];                                                                      \
    _Pragma("unroll") for (int w = 1; w < WAVES; ++w) sum += rb_[w * 64 + lane];                \
    const int lc_ = ((tile) - t0) * 16 + lq * 4;                                                \
    float4 rv = *(const float4*)&r_s[lr * EC + lc_];                                            \
    const float4 bs_ = *(const float4*)&v_s[lc_];                                               \
    if (has_ln) {                                                                               \
      const float4 gg_ = *(const float4*)&v_s[EC + lc_], hh_ = *(const float4*)&v_s[2 * EC + lc_]; \
      rv.x = (rv.x - mu) * rstd * gg_.x + hh_.x; rv.y = (rv.y - mu) * rstd * gg_.y + hh_.y;     \
      rv.z = (rv.z - mu) * rstd * gg_.z + hh_.z; rv.w = (rv.w - mu) * rstd * gg_.w + hh_.w;     \
    }                                                                                           \
    float v[4] = {sum[0] + bs_.x, sum[1] + bs_.y, sum[2] + bs_.z, sum[3] + bs_.w};              \
    if (e.relu) { _Pragma("unroll") for (int r = 0; r < 4; ++r) v[r] = fmaxf(v[r], 0.f); }      \
    v[0] += rv.x; v[1] += rv.y; v[2] += rv.z; v[3] += rv.w;                                     \
    const int n = (tile) * 16 + lq * 4;                                                         \
    if (lr < p.M) {                                                                             \
      if (e.Yf) *(float4*)(e.Yf + g * e.yf_g + (long)lr * e.ldyf + n) = make_float4(v[0], v[1], v[2], v[3]); \
      if (e.Ya) *(uint2*)((bf16_t*)e.Ya + g * e.ya_g + (long)lr * e.ldya + n) = make_uint2(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3])); \
    }                                                                                           \
  }
#define ST_MULT(A)                                                                              \
  {                                                                                             \
    f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};                                                      \
    __builtin_amdgcn_sched_barrier(0);                                                          \
    _Pragma("unroll") for (int i0 = 0; i0 < U; i0 += 4) {      /* four operand reads at a time: registers */ \
      uint4 bb_[4];                                                                             \
      _Pragma("unroll") for (int i = 0; i < 4; ++i) bb_[i] = *(const uint4*)(xrow + (wave + WAVES * (i0 + i)) * 32); \
      _Pragma("unroll") for (int i = 0; i < 4; ++i)                                             \
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A[i0 + i]), __builtin_bit_cast(bf16x8, bb_[i]), acc, 0, 0, 0); \
      __builtin_amdgcn_sched_barrier(0);                                                        \
    }                                                                                           \
    red[(it & 1) * (WAVES * 64) + wave * 64 + lane] = acc;                                      \
  }
  // state "X holds tile t": its weights are in flight or here, the partial sums of tile t - 1 (if any) wait in
  // red[(it - 1) & 1].  The first pass (it == 0) also moves the small operands to LDS; X and the small operands were
  // requested before any weights, so they are complete once at most the weight loads issued since are outstanding.
#define ST_ENTER(younger)                                                                       \
    if (it == 0) { ST_WAIT_VM(younger); ST_SMALL_TO_LDS() }                                     \
    __syncthreads();                                                                            \
    if (it == 0) { if (has_ln) row_stats(st_s, e.lnR_K, e.lnR_eps, lane, mu, rstd); }           \
    else ST_FINISH(t - 1, it - 1)
#define ST_STEP(X, Y)                                                                           \
  {                                                                                             \
    ST_LOADW(Y, t + 1)                                                                          \
    ST_ENTER(32)                                                                                \
    ST_MULT(X)                                                                                  \
    ++it; ++t;                                                                                  \
  }
#define ST_LAST(X)                                                                              \
  {                                                                                             \
    ST_ENTER(16)                                                                                \
    ST_MULT(X)                                                                                  \
    __syncthreads();                                                                            \
    ST_FINISH(t, it)                                                                            \
  }
  int t = t0;
  ST_LOADW(a_cur, t0)
  while (t + 2 < t1) {
    ST_STEP(a_cur, a_nxt)
    ST_STEP(a_nxt, a_cur)
  }
  if (t + 1 == t1) {
    ST_LAST(a_cur)
  } else {
    ST_STEP(a_cur, a_nxt)
    ST_LAST(a_nxt)
  }
#undef ST_ENTER
#undef ST_STEP
#undef ST_LAST
#undef ST_MULT
#undef ST_FINISH
#undef ST_WAIT_VM
#undef ST_SMALL_TO_LDS
#undef ST_LOADW
}

// ---------------------------------------------------------------------------------------
// Streaming vocabulary projection + arg-max for a block of 17 .. 128 rows (the k x k score rows of one
// sentence): K = 512 or 1024, N a multiple of 16.  Grid (GX, row blocks of 64), 512 threads, one
// workgroup per CU.
//   * the workgroup's rows of X (up to 16 * MT = 64, bf16) go global -> LDS once (direct loads,
//     rows padded by 16 bytes against bank conflicts)
//   * a workgroup owns the contiguous column tiles [t0, t1); its 8 waves take them in turn (wave w:
//     t0 + w, t0 + w + 8, ...), NT at a time.  A wave multiplies whole column tiles by itself (no
//     partial sums, no barrier after the prologue): it streams their weights in units of 16 loads
//     (16 / NT k-steps of NT tiles) through two register buffers that take turns, the next unit
//     in flight while one is multiplied against the MT row tiles read from LDS (with NT = 2 one
//     LDS read feeds two MFMAs: half the LDS traffic); k ascends within one accumulator, as in the
//     LDS-staged GEMM, so both give the same bits.  UPT = K / 32 * NT / 16 units per group of NT tiles.
//     A wave with an odd number of tiles repeats its last tile as the partner (same keys again).
//   * each wave keeps a running best key per row; the waves' keys meet in LDS at the end and
//     one 64-bit atomic max per row and workgroup goes to keys[]
// Dynamic LDS: 8 * 16 * MT * 8 bytes (keys) + rows * (K + 8) * 2 bytes (X).
template <int MT, int NT, int UPT, bool STREAM>
__global__ __launch_bounds__(512) void stream_vocab_kernel(GemmP p, unsigned long long* keys, float* logits) {
  constexpr int WAVES = 8, BM = 16 * MT, UK = 16 / NT;      // UK k-steps per unit
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  unsigned long long* wb = (unsigned long long*)smem_raw;  // [WAVES][BM]
  bf16_t* xs = (bf16_t*)(smem_raw + WAVES * BM * 8);
  const int ldxs = p.K + 8;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int lr = lane & 15, lq = lane >> 4;
  const int ntiles = p.N >> 4, ksteps = p.K >> 5;          // ksteps == UK * UPT
  const int m0 = blockIdx.y * BM;
  const int nrows = min(BM, p.M - m0);
  const int t0 = (int)(blockIdx.x * (unsigned)ntiles / gridDim.x), t1 = (int)((blockIdx.x + 1) * (unsigned)ntiles / gridDim.x);
  {   // X: whole wave-loads of 64 pieces (512 columns) inside one row
    const bf16_t* xg = (const bf16_t*)p.X + (long)m0 * p.ldx;
    const int parts = p.K >> 9;                            // 512-column parts per row
#pragma unroll
    for (int i = 0; i < 4 * MT; ++i) {                     // 16 * MT rows * (at most) 2 parts / 8 waves
      const int wl = i * WAVES + wave;
      const int row = wl / parts, part = wl % parts;
      if (row < nrows)
        __builtin_amdgcn_global_load_lds((const void __attribute__((address_space(1)))*)(xg + (long)row * p.ldx + part * 512 + lane * 8),
                                         (void __attribute__((address_space(3)))*)(xs + row * ldxs + part * 512), 16, 0, 0);
    }
  }
  const char* Wg = (const char*)p.W;
  const unsigned loff = lane * 16;
  // this wave's tiles: t0 + wave + 8 * j, j < ntw, in groups of NT; unit u = (group u / UPT, k-steps UK * (u % UPT) .. + UK)
  const int ntw = t0 + wave < t1 ? (t1 - t0 - wave + WAVES - 1) / WAVES : 0;
  const int NU = (ntw + NT - 1) / NT * UPT;
  uint4 a0[16], a1[16];
#define SV_TILE(u, n) (t0 + wave + WAVES * (((u) / UPT) * NT + (n) < ntw ? ((u) / UPT) * NT + (n) : ntw - 1))
#define SV_LOADU(dst, u)                                                                        \
  _Pragma("unroll") for (int n = 0; n < NT; ++n) {                                              \
    const char* wp_ = Wg + ((long)SV_TILE(u, n) * ksteps + UK * ((u) % UPT)) * 1024;            \
    _Pragma("unroll") for (int i = 0; i < UK; ++i) {                                            \
      if (STREAM) dst[n * UK + i] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_nt*)(wp_ + i * 1024 + loff))); \
      else dst[n * UK + i] = *(const uint4*)(wp_ + i * 1024 + loff);                            \
    }                                                                                           \
  }
#define SV_WAIT_VM(n) __builtin_amdgcn_s_waitcnt(((n) & 15) | (7 << 4) | (15 << 8) | (((n) >> 4) << 14))
  if (NU > 0) {
    SV_LOADU(a0, 0)
    SV_WAIT_VM(16);                              // X was requested before the 16 weight loads
  } else {
    SV_WAIT_VM(0);
  }
  __syncthreads();
  const bf16_t* xrow[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int r = t * 16 + lr;
    xrow[t] = xs + (r < nrows ? r : nrows - 1) * ldxs + lq * 8;
  }
  f32x4 acc[MT][NT];
  unsigned long long best[MT];
#pragma unroll
  for (int t = 0; t < MT; ++t) best[t] = 0ull;
  // one unit: UK k-steps of NT column tiles against the MT row tiles
#define SV_MULT(A, u)                                                                           \
  {                                                                                             \
    const int part_ = (u) % UPT;                                                                \
    if (part_ == 0) {                                                                           \
      _Pragma("unroll") for (int t = 0; t < MT; ++t)                                            \
        _Pragma("unroll") for (int n = 0; n < NT; ++n) acc[t][n] = f32x4{0.f, 0.f, 0.f, 0.f};   \
    }                                                                                           \
    __builtin_amdgcn_sched_barrier(0);                                                          \
    _Pragma("unroll") for (int i0 = 0; i0 < UK; i0 += 2) {                                      \
      uint4 bb_[2][MT];                                                                         \
      _Pragma("unroll") for (int i = 0; i < 2; ++i)                                             \
        _Pragma("unroll") for (int t = 0; t < MT; ++t) bb_[i][t] = *(const uint4*)(xrow[t] + (part_ * UK + i0 + i) * 32); \
      _Pragma("unroll") for (int i = 0; i < 2; ++i)                                             \
        _Pragma("unroll") for (int t = 0; t < MT; ++t)                                          \
          _Pragma("unroll") for (int n = 0; n < NT; ++n)                                        \
            acc[t][n] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A[n * UK + i0 + i]), __builtin_bit_cast(bf16x8, bb_[i][t]), acc[t][n], 0, 0, 0); \
      __builtin_amdgcn_sched_barrier(0);                                                        \
    }                                                                                           \
    if (part_ == UPT - 1) {                                                                     \
      _Pragma("unroll") for (int n = 0; n < NT; ++n) {                                          \
        const int n_ = SV_TILE(u, n) * 16 + lq * 4;                                             \
        _Pragma("unroll") for (int t = 0; t < MT; ++t) {                                        \
          _Pragma("unroll") for (int r = 0; r < 4; ++r) {                                       \
            const unsigned long long key_ = argmax_key(acc[t][n][r], (unsigned)(n_ + r));       \
            best[t] = key_ > best[t] ? key_ : best[t];                                          \
          }                                                                                     \
          const int m_ = m0 + t * 16 + lr;                                                      \
          if (logits && m_ < p.M) *(float4*)(logits + (long)m_ * p.N + n_) = make_float4(acc[t][n][0], acc[t][n][1], acc[t][n][2], acc[t][n][3]); \
        }                                                                                       \
      }                                                                                         \
    }                                                                                           \
  }
  int u = 0;
  while (u + 2 < NU) {
    SV_LOADU(a1, u + 1)
    SV_MULT(a0, u)
    SV_LOADU(a0, u + 2)
    SV_MULT(a1, u + 1)
    u += 2;
  }
  if (NU - u == 1) {
    SV_MULT(a0, u)
  } else if (NU - u == 2) {
    SV_LOADU(a1, u + 1)
    SV_MULT(a0, u)
    SV_MULT(a1, u + 1)
  }
#undef SV_MULT
#undef SV_WAIT_VM
#undef SV_LOADU
#undef SV_TILE
  // lanes l, l^16, l^32, l^48 hold the same rows
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    unsigned long long b = best[t];
    unsigned long long o = __shfl_xor(b, 16, 64); b = o > b ? o : b;
    o = __shfl_xor(b, 32, 64); b = o > b ? o : b;
    if (lane < 16) wb[wave * BM + t * 16 + lane] = b;
  }
  __syncthreads();
  if (tid < nrows) {
    unsigned long long b = wb[tid];
#pragma unroll
    for (int w = 1; w < WAVES; ++w) { const unsigned long long o = wb[w * BM + tid]; b = o > b ? o : b; }
    if (b != 0ull) atomicMax(&keys[m0 + tid], b);
  }
}

// 16 bytes per lane from global memory (base, the same for the whole wave, + the lane's byte offset) straight into LDS:
// lane l's piece lands at lds_base + 16 l (lds_base: the same for the whole wave).  Issued from inline assembly on purpose:
// behind the compiler's builtin for this instruction every later LDS read of the kernel is ordered after ALL outstanding
// loads (s_waitcnt vmcnt(0) ahead of the first read of each chunk), so nothing stayed in flight across the matrix
// instructions.  The kernel waits for these loads itself (s_waitcnt vmcnt(n) + workgroup barrier) before reading.
__device__ __forceinline__ void lds_dma16(const void* base, unsigned byte_off, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
               :: "s"(lds_base), "v"(byte_off), "s"(base) : "memory");
}
__device__ __forceinline__ unsigned lds_address(const void* p) {
  return (unsigned)(unsigned long long)(const __attribute__((address_space(3))) void*)p;
}

// ---------------------------------------------------------------------------------------
// "ldsx" GEMM: BM = 16*MT rows x BN = 64*NT columns per workgroup, K walked in chunks of KC.
// Wave w owns column tiles (4*blockIdx.x + w)*NT .. +NT and streams their weight tiles from
// global memory into registers one chunk ahead (KC/32 * NT fragments in flight per wave).  The
// BM x KC activation chunk goes global -> LDS directly (global_load_lds_dwordx4, no staging
// registers), double buffered.  Such a load writes 64 consecutive 16-byte slots per wave, so
// rows cannot be padded; instead the 16-byte segment index within a row is XOR-ed with
// (row & 7), which spreads the MFMA operand reads of a wave evenly over the LDS banks.
// Requires K % KC == 0, KC % 64 == 0 (DEEP tiles: K % 128 == 0).  Dynamic LDS: ldsx_lds_bytes() (2 or 3 buffers of
// XI * 4096 bytes).
// Two workgroups share a CU whenever the accumulators (4*MT*NT registers), the two weight chunks
// (8*NT*KC/32) and the operand fragments (4*MT) leave room for it in half the register file: the
// second wave per SIMD covers the LDS and memory latencies of the first.
template <int MT, int NT, int KC>
constexpr int ldsx_regs() { return 4 * MT * NT + 8 * NT * (KC / 32) + 4 * MT + 40; }
template <int MT, int NT, int KC>
constexpr int ldsx_waves_min() { return ldsx_regs<MT, NT, KC>() <= 272 ? 2 : 1; }
template <int MT, int NT, int KC>
constexpr int ldsx_waves_max() { return ldsx_regs<MT, NT, KC>() <= 168 ? 4 : ldsx_waves_min<MT, NT, KC>(); }

// Large tiles (64 or more rows, 256 columns, chunks of 64) keep more in flight (DEEP): four 32-deep steps of weights in
// registers, each requested again right after the step that used them (what a chunk waits for is the slowest of its ~100
// memory requests, and one in seven misses the L2), three activation buffers, and the LDS reads of one half of a step's
// row tiles overlap the matrix instructions of the other half.  An even number of chunks (K % 128 == 0; the host's tile
// rule sees to it: a third copy of the chunk for an odd tail spilled registers).
// On the 3200 x 32768 x 1024 vocabulary projection: 264 us with the compiler's builtin for the direct loads, 216 us with
// those loads and their waits issued by hand and all LDS reads of a step ahead of its matrix instructions, 196 us as
// DEEP.  Smaller tiles measured no faster as DEEP (the batch-32 step 0.780 ms against 0.760 ms: they lose a workgroup
// per CU to the third buffer), the 64 x 128 tiles of the heads' output layers the same (0.759 ms).
template <int MT, int NT, int KC>
constexpr bool ldsx_deep() { return NT == 4 && KC == 64 && MT >= 4; }
template <int MT, int NT, int KC>
constexpr size_t ldsx_lds_bytes() { return (size_t)(ldsx_deep<MT, NT, KC>() ? 3 : 2) * ((16 * MT * (KC / 8) + 255) / 256) * 4096; }

// XLN (one group, no split-K, K <= 1024): X = LayerNorm(ln.x) of the fp32 residual stream.  The producer of ln.x left per
// 64-column block and row the sum and sum of squares of its values in ln.stats[(block * M + row) * 2] (store_tiles); the
// workgroup adds them for its rows, and every activation chunk goes global (fp32) -> registers -> normalised -> bf16 ->
// LDS, in the layout the direct loads would have produced.  Saves the LayerNorm kernel and its round trip through memory.
// STATS: store_tiles also writes the LayerNorm statistics of the output (e.stats_out).
// ROWAFF (one group, no split-K, K <= 1024, BM <= 64): LayerNorm folded into the weights; mu / rstd of the rows from the
// producer's partial statistics (requested before everything else, reduced while the first chunk arrives), applied in
// the epilogue.  X comes through the direct loads like any bf16 operand: no LayerNorm kernel and no normalisation here.
template <int MT, int NT, int KC, bool ARGMAX, bool XLN, bool STATS, bool ROWAFF = false>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(ldsx_waves_min<MT, NT, KC>(), ldsx_waves_max<MT, NT, KC>()))) void gemm_ldsx_kernel(GemmP p, Epi e, unsigned long long* keys, float* logits, LnP ln) {
  constexpr int BM = 16 * MT, KS = KC / 32, SEG = KC / 8;
  static_assert(!ROWAFF || (BM <= 64 && !XLN && !ARGMAX), "row statistics: one pass over at most 64 rows");
  __shared__ float2 ra_part[ROWAFF ? 4 * 64 : 1];
  __shared__ float2 ra_ms[ROWAFF ? 64 : 1];
  constexpr int XI = (BM * SEG + 255) / 256;       // direct-to-LDS loads per thread per chunk
  constexpr int BUF = XI * 256 * 8;                // bf16 elements per buffer (whole wave-loads)
  extern __shared__ __attribute__((aligned(16))) unsigned char smem_raw[];
  bf16_t* xs0 = (bf16_t*)smem_raw;
  bf16_t* xs1 = xs0 + BUF;
  const int tid = threadIdx.x, lane = tid & 63, wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int g = p.ksplit > 1 ? 0 : blockIdx.z;
  const int ntiles = p.N >> 4, ksteps = p.K >> 5;
  const int nchunks = p.lx.nchunks;                                   // chunks of this K slice (K / KC / slices, from the host)
  const int cbase = p.ksplit > 1 ? blockIdx.z * nchunks : 0;
  int bx, by;                                    // (the map: bpd_tile_map.h)
  ldsx_tile_of(p.lx, gridDim.x, gridDim.y, blockIdx.x, blockIdx.y, blockIdx.z, g, by, bx);
  const int m0 = by * BM;
  const int nt0 = (bx * 4 + wave) * NT;
  const int lr = lane & 15, lq = lane >> 4;
  const bf16_t* X = (const bf16_t*)p.X + g * p.x_g;
  const bf16_t* W = (const bf16_t*)p.W + g * p.w_g;
  const uint4* wt[NT];
#pragma unroll
  for (int u = 0; u < NT; ++u) {
    int tile = nt0 + u;
    tile = tile < ntiles ? tile : ntiles - 1;
    wt[u] = (const uint4*)W + (long)tile * ksteps * 64 + lane;
  }
  // slot i*256 + tid of a buffer holds row = slot / SEG, segment (slot % SEG) ^ (row & 7)
  unsigned xoff[XI];
#pragma unroll
  for (int i = 0; i < XI; ++i) {
    const int slot = tid + 256 * i;
    const int r = slot / SEG;
    int row = m0 + r;
    row = row < p.M ? row : p.M - 1;
    xoff[i] = (row * p.ldx + (((slot % SEG) ^ (r & 7)) * 8)) * 2;      // bytes
  }
#define BPD_X_TO_LDS(buf, chunk)                                                            \
  _Pragma("unroll") for (int i = 0; i < XI; ++i)                                            \
    lds_dma16(X + (chunk) * KC, xoff[i], lds_address((buf) + (i * 256 + wave * 64) * 8));
  if constexpr (XLN) {
    // ---- LayerNorm-fused variant: activations through registers
    static_assert(256 % SEG == 0, "a thread keeps its 16-byte segment across its rows");
    __shared__ float2 part_s[4][64];
    __shared__ float2 ms_s[BM];
    static_assert(BM <= 64, "one pass of the statistics reduction");
    constexpr int RPI = 256 / SEG;               // rows between a thread's consecutive slots
    const int seg = tid % SEG, rbase = tid / SEG;
    const float* xp[XI];
    int lo[XI], rcl[XI];
#pragma unroll
    for (int i = 0; i < XI; ++i) {
      const int r = rbase + RPI * i;             // may pass BM when BM * SEG is not a multiple of 256: never read back
      rcl[i] = r < BM ? r : BM - 1;
      int row = m0 + rcl[i]; row = row < p.M ? row : p.M - 1;
      xp[i] = ln.x + (long)row * p.K + seg * 8;
      lo[i] = (r * SEG + (seg ^ (r & 7))) * 8;
    }
    uint4 a0[KS][NT], a1[KS][NT];
    f32x4 acc[MT][NT];
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int u = 0; u < NT; ++u) acc[t][u] = f32x4{0.f, 0.f, 0.f, 0.f};
    float4 xa[XI][2], ga[2], ba[2];
#define BPD_LOAD_X(chunk)                                                                    \
    {                                                                                        \
      _Pragma("unroll") for (int i = 0; i < XI; ++i) {                                       \
        xa[i][0] = *(const float4*)(xp[i] + (chunk) * KC); xa[i][1] = *(const float4*)(xp[i] + (chunk) * KC + 4); \
      }                                                                                      \
      ga[0] = *(const float4*)(ln.g + (chunk) * KC + seg * 8); ga[1] = *(const float4*)(ln.g + (chunk) * KC + seg * 8 + 4); \
      ba[0] = *(const float4*)(ln.b + (chunk) * KC + seg * 8); ba[1] = *(const float4*)(ln.b + (chunk) * KC + seg * 8 + 4); \
    }
#define BPD_NORM1(v, gq, bq, i) ((v - mu[i]) * rs[i] * gq + bq)
#define BPD_NORM_STORE(buf)                                                                  \
    _Pragma("unroll") for (int i = 0; i < XI; ++i) {                                         \
      const unsigned w0 = pack_bf16(BPD_NORM1(xa[i][0].x, ga[0].x, ba[0].x, i), BPD_NORM1(xa[i][0].y, ga[0].y, ba[0].y, i)); \
      const unsigned w1 = pack_bf16(BPD_NORM1(xa[i][0].z, ga[0].z, ba[0].z, i), BPD_NORM1(xa[i][0].w, ga[0].w, ba[0].w, i)); \
      const unsigned w2 = pack_bf16(BPD_NORM1(xa[i][1].x, ga[1].x, ba[1].x, i), BPD_NORM1(xa[i][1].y, ga[1].y, ba[1].y, i)); \
      const unsigned w3 = pack_bf16(BPD_NORM1(xa[i][1].z, ga[1].z, ba[1].z, i), BPD_NORM1(xa[i][1].w, ga[1].w, ba[1].w, i)); \
      *(uint4*)((buf) + lo[i]) = make_uint4(w0, w1, w2, w3);                                 \
    }
#define BPD_LOAD_WX(dst, chunk)                                                              \
    _Pragma("unroll") for (int s = 0; s < KS; ++s)                                           \
      _Pragma("unroll") for (int u = 0; u < NT; ++u) dst[s][u] = wt[u][(long)((chunk) * KS + s) * 64];
    // activations are requested before the weights: waiting for them leaves the weights in flight
#define BPD_CHUNK_X(AC, AL, xc, xl, c)                                                       \
    {                                                                                        \
      const int cl = (c) + 1 < nchunks ? (c) + 1 : nchunks - 1;                              \
      BPD_LOAD_X(cl)                                                                         \
      BPD_LOAD_WX(AL, cl)                                                                    \
      __builtin_amdgcn_sched_barrier(0);                                                     \
      _Pragma("unroll") for (int s = 0; s < KS; ++s) {                                       \
        uint4 b[MT];                                                                         \
        _Pragma("unroll") for (int t = 0; t < MT; ++t)                                       \
          b[t] = *(const uint4*)((xc) + (t * 16 + lr) * KC + (((s * 4 + lq) ^ (lr & 7)) * 8)); \
        _Pragma("unroll") for (int t = 0; t < MT; ++t)                                       \
          _Pragma("unroll") for (int u = 0; u < NT; ++u)                                     \
            acc[t][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, AC[s][u]), \
                                                                __builtin_bit_cast(bf16x8, b[t]), acc[t][u], 0, 0, 0); \
      }                                                                                      \
      __builtin_amdgcn_sched_barrier(0);                                                     \
      BPD_NORM_STORE(xl)                                                                     \
      __syncthreads();                                                                       \
    }
    // one round trip for everything the first chunk needs: the statistics, the first activations and weights
    float mu[XI], rs[XI];
    constexpr bool XPREF = MT * NT <= 3;
    float4 xpre_b[XPREF ? NT : 1], xpre_r[XPREF ? MT * NT : 1];
    const bool xpre = XPREF && e.pre_epi != 0;
    {
      // (one partial per 64-column block; 16 rows: thread = (block tid / 16, row tid % 16): one load per thread)
      constexpr int RL = MT == 1 ? 1 : 4;
      const int tiles = p.K >> 6;                // 64-column blocks of the producer, <= 16
      int row = m0 + (MT == 1 ? (tid & 15) : lane); row = row < p.M ? row : p.M - 1;
      float2 pv[RL];
#pragma unroll
      for (int i = 0; i < RL; ++i) {             // branch-free: all loads in flight together
        const int t = MT == 1 ? (tid >> 4) + 16 * i : wave + 4 * i;
        pv[i] = ((const float2*)ln.stats)[(long)(t < tiles ? t : 0) * p.M + row];
      }
      BPD_LOAD_X(0)
      BPD_LOAD_WX(a0, 0)
      if (xpre) {                                // bias and residual of the epilogue ride along (Epi::pre_epi)
#pragma unroll
        for (int u = 0; u < NT; ++u) {
          const int n = (nt0 + u < ntiles ? nt0 + u : ntiles - 1) * 16 + lq * 4;
          xpre_b[u] = *(const float4*)(e.bias + n);
#pragma unroll
          for (int t = 0; t < MT; ++t) {
            int m = m0 + t * 16 + lr; m = m < p.M ? m : p.M - 1;
            xpre_r[t * NT + u] = *(const float4*)(e.R + (long)m * e.ldr + n);
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      float sq = 0.f, qq = 0.f;
#pragma unroll
      for (int i = 0; i < RL; ++i) {
        const float w = (MT == 1 ? (tid >> 4) + 16 * i : wave + 4 * i) < tiles ? 1.f : 0.f;
        sq = fmaf(w, pv[i].x, sq); qq = fmaf(w, pv[i].y, qq);
      }
      (&part_s[0][0])[MT == 1 ? tid : wave * 64 + lane] = make_float2(sq, qq);      // [class][16 rows] or [wave][64 rows]
      __syncthreads();
      if (tid < BM) {
        constexpr int NP = MT == 1 ? 16 : 4, PS = MT == 1 ? 16 : 64;
        float S = part_s[0][tid].x, Q = part_s[0][tid].y;
#pragma unroll
        for (int w = 1; w < NP; ++w) { S += (&part_s[0][0])[w * PS + tid].x; Q += (&part_s[0][0])[w * PS + tid].y; }
        const float mean = S / p.K;
        const float var = fmaxf(Q / p.K - mean * mean, 0.f);
        ms_s[tid] = make_float2(mean, 1.0f / sqrtf(var + ln.eps));
      }
      __syncthreads();
#pragma unroll
      for (int i = 0; i < XI; ++i) { const float2 ms = ms_s[rcl[i]]; mu[i] = ms.x; rs[i] = ms.y; }
    }
    BPD_NORM_STORE(xs0)
    __syncthreads();
    for (int c = 0; c < nchunks; c += 2) {
      BPD_CHUNK_X(a0, a1, xs0, xs1, c)
      if (c + 1 >= nchunks) break;
      BPD_CHUNK_X(a1, a0, xs1, xs0, c + 1)
    }
#undef BPD_CHUNK_X
#undef BPD_LOAD_WX
#undef BPD_NORM_STORE
#undef BPD_NORM1
#undef BPD_LOAD_X
    if (nt0 >= ntiles) return;
    store_tiles<MT, NT, STATS>(e, g, acc, m0, nt0, ntiles, p.M, lane, nullptr, nullptr, nullptr, XPREF ? xpre_b : nullptr, XPREF ? xpre_r : nullptr, smem_raw + wave * 2048);
    return;
  }
  // The direct-to-LDS loads of the loop are issued from inline assembly (lds_dma16) and waited for by hand (s_waitcnt
  // vmcnt(n): at most the n youngest loads of this wave still outstanding; loads complete in issue order).  Through the
  // compiler's builtin every later LDS read is ordered behind ALL outstanding loads, whichever buffer they fill, which ends
  // in vmcnt(0) ahead of each chunk's first read and leaves nothing in flight across the matrix instructions.  The weight
  // loads stay ordinary loads: the compiler's own waits for them count only the loads it knows of, so with the direct
  // loads in the queue they cover a few more loads than needed (never fewer): each weight request is therefore issued
  // AHEAD of the activation request of its chunk, which keeps what is covered to loads of about the same age.
  //
  // Plain tiles: the chunk being multiplied and the next one are in use / in flight, weights in two register sets that
  // take turns, activations in two LDS buffers.
  // DEEP tiles: four 32-deep steps of weights in registers, each requested again (two chunks ahead) right after the step
  // that used them; three activation buffers.
  constexpr bool DEEP = ldsx_deep<MT, NT, KC>();
  uint4 a0[KS][NT], a1[KS][NT];
  f32x4 acc[MT][NT];
#pragma unroll
  for (int t = 0; t < MT; ++t)
#pragma unroll
    for (int u = 0; u < NT; ++u) acc[t][u] = f32x4{0.f, 0.f, 0.f, 0.f};
#define BPD_LOAD_WS(dst, step)                                                               \
  _Pragma("unroll") for (int u = 0; u < NT; ++u) dst[u] = wt[u][(long)(step) * 64];
#define BPD_LOAD_W(dst, chunk)                                                               \
  _Pragma("unroll") for (int s = 0; s < KS; ++s) BPD_LOAD_WS(dst[s], (chunk) * KS + s)
#define BPD_WAIT_VM(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")
  // small tiles: bias and residual of the epilogue are requested first
  constexpr bool PREF = !ARGMAX && MT * NT <= 3;
  float4 pre_b[PREF ? NT : 1], pre_r[PREF ? MT * NT : 1];
  const bool pre = PREF && e.pre_epi != 0;       // (uniform)
  if constexpr (PREF) {
    if (pre) {
#pragma unroll
      for (int u = 0; u < NT; ++u) {
        const int n = (nt0 + u < ntiles ? nt0 + u : ntiles - 1) * 16 + lq * 4;
        pre_b[u] = *(const float4*)(e.bias + g * e.bias_g + n);
#pragma unroll
        for (int t = 0; t < MT; ++t) {
          int m = m0 + t * 16 + lr; m = m < p.M ? m : p.M - 1;
          pre_r[t * NT + u] = *(const float4*)(e.R + g * e.r_g + (long)m * e.ldr + n);
        }
      }
    }
  }
  // row statistics (one partial per 64-column block): RL loads per thread.  16 rows: thread = (block tid / 16, row
  // tid % 16); more rows: lane = row, blocks wave + 4 i
  constexpr int RL = MT == 1 ? 1 : 4;
  float2 rpv[ROWAFF ? RL : 1];
  float4 ra_c4[NT], ra_d4[NT];
  if constexpr (ROWAFF) {
    int row = m0 + (MT == 1 ? (tid & 15) : lane); row = row < p.M ? row : p.M - 1;
    const int tiles = p.K >> 6;                  // 64-column blocks of the producer, <= 16
#pragma unroll
    for (int i = 0; i < RL; ++i) {
      const int t = MT == 1 ? (tid >> 4) + 16 * i : wave + 4 * i;
      rpv[i] = ((const float2*)e.ra_stats)[(long)(t < tiles ? t : 0) * p.M + row];
    }
#pragma unroll
    for (int u = 0; u < NT; ++u) {               // column operands of the epilogue, for this lane's four columns per tile
      const int tile = nt0 + u < ntiles ? nt0 + u : ntiles - 1;
      ra_c4[u] = *(const float4*)(e.ra_c + tile * 16 + lq * 4);
      ra_d4[u] = *(const float4*)(e.ra_d + tile * 16 + lq * 4);
    }
  }
  const bf16_t* xa = xs0;                        // DEEP: the activation buffers take turns (xa: multiplied, xb: next, xf: filling)
  const bf16_t* xb = xs1;
  bf16_t* xf = xs1 + (DEEP ? BUF : 0);
  const int c1 = cbase + (1 < nchunks ? 1 : 0);
  if constexpr (DEEP) {                          // two chunks up front; both have landed when the loop starts
    BPD_X_TO_LDS(xs0, cbase)
    BPD_LOAD_W(a0, cbase)
    BPD_X_TO_LDS(xs1, c1)
    BPD_LOAD_W(a1, c1)
    BPD_WAIT_VM(0);
  } else {
    BPD_LOAD_W(a0, cbase)
    BPD_X_TO_LDS(xs0, cbase)
    BPD_WAIT_VM(0);
  }
  if constexpr (ROWAFF) {
    const int tiles = p.K >> 6;
    float sq = 0.f, qq = 0.f;
#pragma unroll
    for (int i = 0; i < RL; ++i) {
      const float w = (MT == 1 ? (tid >> 4) + 16 * i : wave + 4 * i) < tiles ? 1.f : 0.f;
      sq = fmaf(w, rpv[i].x, sq); qq = fmaf(w, rpv[i].y, qq);
    }
    ra_part[MT == 1 ? tid : wave * 64 + lane] = make_float2(sq, qq);      // [class][16 rows] or [wave][64 rows]
  }
  __syncthreads();
  if constexpr (ROWAFF) {                        // read back in the epilogue, many barriers later
    if (tid < BM) {
      constexpr int NP = MT == 1 ? 16 : 4, PS = MT == 1 ? 16 : 64;
      float S = ra_part[tid].x, Q = ra_part[tid].y;
#pragma unroll
      for (int w = 1; w < NP; ++w) { S += ra_part[w * PS + tid].x; Q += ra_part[w * PS + tid].y; }
      const float mean = S / p.K;
      const float var = fmaxf(Q / p.K - mean * mean, 0.f);
      ra_ms[tid] = make_float2(mean, 1.0f / sqrtf(var + e.ra_eps));
    }
  }
  // one 32-deep step: the MT activation fragments from LDS (all requested before the first matrix instruction, which
  // then waits for its own fragment only), MT x NT matrix instructions
#define BPD_XFRAG(xc, s, t) *(const uint4*)((xc) + ((t) * 16 + lr) * KC + ((((s) * 4 + lq) ^ (lr & 7)) * 8))
#define BPD_STEP(A_, xc, s)                                                                  \
  {                                                                                          \
    uint4 b[MT];                                                                             \
    _Pragma("unroll") for (int t = 0; t < MT; ++t) b[t] = BPD_XFRAG(xc, s, t);               \
    _Pragma("unroll") for (int t = 0; t < MT; ++t)                                           \
      _Pragma("unroll") for (int u = 0; u < NT; ++u)                                         \
        acc[t][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A_[u]), \
                                                            __builtin_bit_cast(bf16x8, b[t]), acc[t][u], 0, 0, 0); \
    __builtin_amdgcn_sched_group_barrier(0x100, MT, 0);                                      \
    __builtin_amdgcn_sched_group_barrier(0x008, MT * NT, 0);                                 \
  }
  // Plain chunk c (weights in AC, activations in xc): chunk c + 1 starts moving into AL / xl, chunk c is multiplied, and
  // the workgroup meets once activation chunk c + 1 has landed: its request is the youngest, so that is when nothing is
  // outstanding any more.  The last chunk requests itself again (branch-free).
#define BPD_CHUNK(AC, AL, xc, xl, c)                                                         \
  {                                                                                          \
    const int cl = cbase + ((c) + 1 < nchunks ? (c) + 1 : nchunks - 1);                      \
    BPD_LOAD_W(AL, cl)                                                                       \
    BPD_X_TO_LDS(xl, cl)                                                                     \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    _Pragma("unroll") for (int s = 0; s < KS; ++s) {                                         \
      BPD_STEP(AC[s], xc, s)                                                                 \
      __builtin_amdgcn_sched_barrier(0);                                                     \
    }                                                                                        \
    BPD_WAIT_VM(0);                                                                          \
    __syncthreads();                                                                         \
  }
  // DEEP chunk c (its two steps' weights in A: a0 / a1 in turn; activations in xa).  The row tiles of a step go in two
  // halves: while the matrix instructions of one half are issued the other half's fragments (of the same step, or of the
  // next one) are on their way from LDS.  The first half of the next chunk's first step is requested before this
  // chunk's last half-step, so the workgroup meets there: activation chunk c + 1 has landed by then (younger than its
  // request: the weights of that chunk's second step and this chunk's first refill), and no wave still reads chunk
  // c - 1, whose buffer (xf) chunk c + 2 starts moving into.  A step's weights are requested again (chunk c + 2) once its
  // matrix instructions are issued.  Issue order per chunk: weights of step 0, activations, weights of step 1.
#define BPD_HALF(A_, B_, T0, TN)                                                             \
  _Pragma("unroll") for (int t = 0; t < TN; ++t)                                             \
    _Pragma("unroll") for (int u = 0; u < NT; ++u)                                           \
      acc[T0 + t][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, A_[u]), \
                                                               __builtin_bit_cast(bf16x8, B_[t]), acc[T0 + t][u], 0, 0, 0); \
  __builtin_amdgcn_sched_barrier(0);
#define BPD_READ_LO(xc, s) _Pragma("unroll") for (int t = 0; t < ML; ++t) blo[t] = BPD_XFRAG(xc, s, t); __builtin_amdgcn_sched_barrier(0);
#define BPD_READ_HI(xc, s) _Pragma("unroll") for (int t = 0; t < MH; ++t) bhi[t] = BPD_XFRAG(xc, s, ML + t); __builtin_amdgcn_sched_barrier(0);
#define BPD_CHUNK_DEEP(A, c)                                                                 \
  {                                                                                          \
    const int cl = cbase + ((c) + 2 < nchunks ? (c) + 2 : nchunks - 1);                      \
    _Pragma("unroll") for (int s = 0; s < KS - 1; ++s) {                                     \
      BPD_READ_HI(xa, s)                                                                     \
      BPD_HALF(A[s], blo, 0, ML)                                                             \
      BPD_READ_LO(xa, s + 1)                                                                 \
      BPD_HALF(A[s], bhi, ML, MH)                                                            \
      BPD_LOAD_WS(A[s], cl * KS + s)                                                         \
      __builtin_amdgcn_sched_barrier(0);                                                     \
    }                                                                                        \
    BPD_READ_HI(xa, KS - 1)                                                                  \
    BPD_HALF(A[KS - 1], blo, 0, ML)                                                          \
    BPD_WAIT_VM(KS * NT);                                                                    \
    __syncthreads();                                                                         \
    BPD_X_TO_LDS(xf, cl)                                                                     \
    BPD_READ_LO(xb, 0)                                                                       \
    BPD_HALF(A[KS - 1], bhi, ML, MH)                                                         \
    BPD_LOAD_WS(A[KS - 1], cl * KS + KS - 1)                                                 \
    __builtin_amdgcn_sched_barrier(0);                                                       \
    { const bf16_t* t_ = xa; xa = xb; xb = xf; xf = (bf16_t*)t_; }                           \
  }
  if constexpr (DEEP) {
    static_assert(KS * NT <= 63, "vmcnt range");
    constexpr int ML = MT / 2, MH = MT - ML;
    uint4 blo[ML > 0 ? ML : 1], bhi[MH];
    BPD_READ_LO(xa, 0)
    for (int c = 0; c < nchunks; c += 2) {       // (an even number of chunks: the host's tile choice sees to it)
      BPD_CHUNK_DEEP(a0, c)
      BPD_CHUNK_DEEP(a1, c + 1)
    }
    BPD_WAIT_VM(0);                              // the last chunks requested themselves again: those copies still land in LDS
    __syncthreads();
  } else {
    int c = 0;
    for (; c + 1 < nchunks; c += 2) {
      BPD_CHUNK(a0, a1, xs0, xs1, c)
      BPD_CHUNK(a1, a0, xs1, xs0, c + 1)
    }
    if (c < nchunks) BPD_CHUNK(a0, a1, xs0, xs1, c)
  }
#undef BPD_READ_HI
#undef BPD_READ_LO
#undef BPD_HALF
#undef BPD_XFRAG
#undef BPD_CHUNK_DEEP
#undef BPD_CHUNK
#undef BPD_STEP
#undef BPD_WAIT_VM
#undef BPD_LOAD_W
#undef BPD_LOAD_WS
#undef BPD_X_TO_LDS
  if (ARGMAX) {
    // per-row best of each wave -> LDS -> one atomic per row and workgroup
    unsigned long long* wb = (unsigned long long*)smem_raw;       // [4][BM], the staging buffers are free now
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const int m = m0 + t * 16 + lr;
      unsigned long long best = 0ull;
#pragma unroll
      for (int u = 0; u < NT; ++u) {
        if (nt0 + u >= ntiles) continue;
        const int n = (nt0 + u) * 16 + (lane >> 4) * 4;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
          const unsigned long long key = argmax_key(acc[t][u][r], (unsigned)(n + r));
          best = key > best ? key : best;
        }
        if (logits && m < p.M)
          *(float4*)(logits + (long)m * p.N + n) = make_float4(acc[t][u][0], acc[t][u][1], acc[t][u][2], acc[t][u][3]);
      }
      unsigned long long o = __shfl_xor(best, 16, 64); best = o > best ? o : best;
      o = __shfl_xor(best, 32, 64); best = o > best ? o : best;
      if (lane < 16) wb[wave * BM + t * 16 + lane] = best;
    }
    __syncthreads();
    if (tid < BM && m0 + tid < p.M) {
      unsigned long long best = wb[tid];
#pragma unroll
      for (int w = 1; w < 4; ++w) { const unsigned long long o = wb[w * BM + tid]; best = o > best ? o : best; }
      if (best != 0ull) atomicMax(&keys[m0 + tid], best);
    }
    return;
  }
  if (nt0 >= ntiles) return;
  if (p.ksplit > 1) {
    float* part = p.part + (long)blockIdx.z * p.M * p.N;
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      const int m = m0 + t * 16 + lr;
      if (m >= p.M) continue;
#pragma unroll
      for (int u = 0; u < NT; ++u) {
        if (nt0 + u >= ntiles) continue;
        *(float4*)(part + (long)m * p.N + (nt0 + u) * 16 + lq * 4) = make_float4(acc[t][u][0], acc[t][u][1], acc[t][u][2], acc[t][u][3]);
      }
    }
    return;
  }
  store_tiles<MT, NT, STATS, ROWAFF>(e, g, acc, m0, nt0, ntiles, p.M, lane, ra_ms, ra_c4, ra_d4, PREF ? pre_b : nullptr, PREF ? pre_r : nullptr, smem_raw + wave * 2048);
}
