// Device code of libbpd: hand-written HIP kernels for gfx950 (CDNA4, 64-wide wavefronts).
//
// Number formats.  "act" tensors (GEMM inputs, K/V caches) are bf16 in BPD_BF16 mode and
// fp32 in BPD_F32 mode; the residual stream, LayerNorm statistics, softmax and all GEMM
// accumulators are fp32.  bf16 values are carried as uint16 bit patterns.
//
// Weight layout in bf16 mode.  A matrix W[K][N] (y = x W) is stored as MFMA operand tiles:
//     Wp[n/16][k/32][lane][e],  lane = 16*((k%32)/8) + n%16,  e = k%8
// so that the 64 lanes of a wavefront fetch one 16x32 tile (1 KiB) with a single fully
// coalesced 16-byte load per lane, directly in the register layout that
// v_mfma_f32_16x16x32_bf16 expects for its first operand.  The weights play the role of the
// MFMA "A" operand (16 output features x 32 k) and the activations are the "B" operand
// (32 k x 16 rows): a block of k <= 16 decoder rows then fills one MFMA tile exactly.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "bpd_tile_map.h"

typedef unsigned short bf16_t;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

__device__ __forceinline__ float bf2f(bf16_t v) { return __uint_as_float(((unsigned)v) << 16); }
__device__ __forceinline__ bf16_t f2bf(float f) {          // round to nearest even
  unsigned u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}
template <typename T> __device__ __forceinline__ float to_f(T v);
template <> __device__ __forceinline__ float to_f<float>(float v) { return v; }
template <> __device__ __forceinline__ float to_f<bf16_t>(bf16_t v) { return bf2f(v); }
template <typename T> __device__ __forceinline__ T from_f(float v);
template <> __device__ __forceinline__ float from_f<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16_t from_f<bf16_t>(float v) { return f2bf(v); }

__device__ __forceinline__ float wave_max(float v) {
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}

// ---------------------------------------------------------------------------------------
// GEMM epilogue shared by the MFMA and the fp32 kernels.
// mode 0:  v = acc (+bias[n]) (ReLU) (+R[m][n]);  Yf[m][n] = v (fp32)  and/or  Ya[m][n] = act(v)
// mode 1:  the N axis is cut into chunks of `dsplit` columns; chunk c = n/dsplit + chunk0
//          c == 0 -> Qf[m][n%dsplit] (fp32),  c == 1 -> Ka,  c == 2 -> Va  (act type) at row
//          (m / rows_per_seq) * cap + (base ? base[m / rows_per_seq] : 0) + m % rows_per_seq
//          (a K/V cache write at the sequence's current length).
struct Epi {
  int mode;
  int relu;
  const float* bias;
  const float* R;  int ldr;
  float* Yf;       int ldyf;
  void* Ya;        int ldya;
  long bias_g, r_g, yf_g, ya_g;      // per-group (blockIdx.z) element offsets
  // skinny kernels only: the residual operand is LayerNorm(R) computed from partial statistics,
  // and/or partial LayerNorm statistics of the result are written (see bpd_gemm.h; the LDS-staged kernel writes them
  // too, with the row count as the stride between column tiles)
  const float* lnR_stats; const float* lnR_g; const float* lnR_b; int lnR_K; float lnR_eps;
  float* stats_out;
  // LDS-staged kernel, LayerNorm folded into the GEMM (ROWAFF): X is the raw bf16 copy of the residual stream, W the
  // weights with the LayerNorm gain multiplied in, and every product is finished per row and column as
  //   rstd[m] * (acc - mu[m] * ra_c[n]) + ra_d[n],   ra_c = column sums of those weights, ra_d = LayerNorm bias . W,
  // with mu / rstd from the partial statistics ra_stats[(tile * M + row) * 2] that the producer of X left
  const float* ra_stats; const float* ra_c; const float* ra_d; float ra_eps;
  // LDS-staged kernel, small tiles (MT * NT <= 3), mode 0, no split over K: bias and residual are fetched at kernel entry
  // instead of in the epilogue (one exposed round trip less).  The host then passes a zero-filled vector for an absent
  // bias (bias_g = 0) or residual (ldr = 0, r_g = 0) so that the loads are unconditional, and sets pre_epi.
  int pre_epi;
  // mode 1
  float* Qf; void* Ka; void* Va;
  int dsplit, chunk0, rows_per_seq, cap;
  const int* base;
};

template <typename ACT>
__device__ __forceinline__ void epi_store(const Epi& e, int g, int m, int n, float v) {
  if (e.mode == 0) {
    if (e.bias) v += e.bias[g * e.bias_g + n];
    if (e.relu) v = fmaxf(v, 0.f);
    if (e.R) v += e.R[g * e.r_g + (long)m * e.ldr + n];
    if (e.Yf) e.Yf[g * e.yf_g + (long)m * e.ldyf + n] = v;
    if (e.Ya) ((ACT*)e.Ya)[g * e.ya_g + (long)m * e.ldya + n] = from_f<ACT>(v);
  } else {
    const int c = n / e.dsplit + e.chunk0;
    const int col = n % e.dsplit;
    if (c == 0) {
      e.Qf[(long)m * e.dsplit + col] = v;
    } else {
      const int b = m / e.rows_per_seq, i = m % e.rows_per_seq;
      const long row = (long)b * e.cap + (e.base ? e.base[b] : 0) + i;
      ACT* dst = (ACT*)(c == 1 ? e.Ka : e.Va);
      dst[row * e.dsplit + col] = from_f<ACT>(v);
    }
  }
}

// Four consecutive columns n .. n+3 (n % 4 == 0, all inside one 16-column tile) of row m, bf16
// activations: the same arithmetic as epi_store with 16-byte loads and 8- / 16-byte stores.
// Needs ldr, ldyf, ldya, dsplit and the per-group offsets to be multiples of 4 (they are model
// dimensions, multiples of 16).
// `fin` receives the stored values (mode 0).
__device__ __forceinline__ void epi_store4f(const Epi& e, int g, int m, int n, const float (&acc)[4], float (&fin)[4]) {
  float v[4] = {acc[0], acc[1], acc[2], acc[3]};
  if (e.mode == 0) {
    if (e.bias) {
      const float4 bs = *(const float4*)(e.bias + g * e.bias_g + n);
      v[0] += bs.x; v[1] += bs.y; v[2] += bs.z; v[3] += bs.w;
    }
    if (e.relu) {
#pragma unroll
      for (int r = 0; r < 4; ++r) v[r] = fmaxf(v[r], 0.f);
    }
    if (e.R) {
      const float4 rv = *(const float4*)(e.R + g * e.r_g + (long)m * e.ldr + n);
      v[0] += rv.x; v[1] += rv.y; v[2] += rv.z; v[3] += rv.w;
    }
    if (e.Yf) *(float4*)(e.Yf + g * e.yf_g + (long)m * e.ldyf + n) = make_float4(v[0], v[1], v[2], v[3]);
    if (e.Ya) *(uint2*)((bf16_t*)e.Ya + g * e.ya_g + (long)m * e.ldya + n) =
                  make_uint2((unsigned)f2bf(v[0]) | ((unsigned)f2bf(v[1]) << 16), (unsigned)f2bf(v[2]) | ((unsigned)f2bf(v[3]) << 16));
    fin[0] = v[0]; fin[1] = v[1]; fin[2] = v[2]; fin[3] = v[3];
  } else {
    const int c = n / e.dsplit + e.chunk0;
    const int col = n % e.dsplit;
    if (c == 0) {
      *(float4*)(e.Qf + (long)m * e.dsplit + col) = make_float4(v[0], v[1], v[2], v[3]);
    } else {
      const int b = m / e.rows_per_seq, i = m % e.rows_per_seq;
      const long row = (long)b * e.cap + (e.base ? e.base[b] : 0) + i;
      bf16_t* dst = (bf16_t*)(c == 1 ? e.Ka : e.Va);
      *(uint2*)(dst + row * e.dsplit + col) =
          make_uint2((unsigned)f2bf(v[0]) | ((unsigned)f2bf(v[1]) << 16), (unsigned)f2bf(v[2]) | ((unsigned)f2bf(v[3]) << 16));
    }
  }
}

__device__ __forceinline__ void epi_store4(const Epi& e, int g, int m, int n, const float (&acc)[4]) {
  float fin[4];
  epi_store4f(e, g, m, n, acc, fin);
}

struct GemmP {
  const void* X; int ldx; long x_g;    // activations [M][K] (act type), per-group offset
  const void* W; long w_g;             // bf16: packed tiles;  fp32: row-major [K][ldw]
  int ldw;
  int M, N, K;
  // split-K (gemm_ldsx_kernel, one group): blockIdx.z = slice of K; the raw fp32 product of slice z
  // goes to part + z*M*N and the consumer (layernorm_kernel) adds the slices in index order
  int ksplit; float* part;
  LdsxMap lx;          // gemm_ldsx_kernel: its workgroup -> tile map and K walk (bpd_tile_map.h; set by the launcher)
};

// ---------------------------------------------------------------------------------------
// bf16 MFMA GEMM.  One workgroup = 4 wavefronts.
//   KS == 4: the 4 waves share NT feature tiles (16 columns each) and split K 4 ways
//            (interleaved 32-wide steps, so neighbouring waves read neighbouring 1 KiB weight
//            tiles); partial sums meet in LDS.  Used when N is small so that N/16 workgroups
//            still spread the weight stream over many CUs.
//   KS == 1: each wave owns NT feature tiles of its own; the workgroup covers 4*NT tiles.
// MT = number of 16-row tiles of X handled by the workgroup (rows m0 .. m0+16*MT).
template <int MT, int NT, int KS>
struct GemmMain {
  f32x4 acc[MT][NT];
  int m0, nt0, lane, wave;
  bool active;

  __device__ __forceinline__ void run(const GemmP& p, f32x4* red /* LDS, KS==4 only */) {
    lane = threadIdx.x & 63;
    wave = threadIdx.x >> 6;
    const int g = blockIdx.z;
    const bf16_t* X = (const bf16_t*)p.X + g * p.x_g;
    const bf16_t* W = (const bf16_t*)p.W + g * p.w_g;
    m0 = blockIdx.y * (16 * MT);
    nt0 = (KS == 4) ? blockIdx.x * NT : (blockIdx.x * 4 + wave) * NT;
    const int ntiles = p.N >> 4, ksteps = p.K >> 5;
    active = nt0 < ntiles;
    const int lr = lane & 15, lk = (lane >> 4) * 8;
#pragma unroll
    for (int t = 0; t < MT; ++t)
#pragma unroll
      for (int u = 0; u < NT; ++u) acc[t][u] = f32x4{0.f, 0.f, 0.f, 0.f};
    const bf16_t* xrow[MT];
#pragma unroll
    for (int t = 0; t < MT; ++t) {
      int r = m0 + t * 16 + lr;
      r = r < p.M ? r : p.M - 1;
      xrow[t] = X + (long)r * p.ldx + lk;
    }
    const uint4* wt[NT];
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      int tile = nt0 + u;
      tile = tile < ntiles ? tile : ntiles - 1;
      wt[u] = (const uint4*)W + (long)tile * ksteps * 64 + lane;
    }
    if (active) {
#pragma unroll 4
      for (int ks = (KS == 4 ? wave : 0); ks < ksteps; ks += KS) {
        uint4 a[NT], b[MT];
#pragma unroll
        for (int u = 0; u < NT; ++u) a[u] = wt[u][(long)ks * 64];
#pragma unroll
        for (int t = 0; t < MT; ++t) b[t] = *(const uint4*)(xrow[t] + ks * 32);
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
          for (int u = 0; u < NT; ++u)
            acc[t][u] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(
                __builtin_bit_cast(bf16x8, a[u]), __builtin_bit_cast(bf16x8, b[t]), acc[t][u], 0, 0, 0);
      }
    }
    if (KS == 4) {
      if (wave > 0) {
#pragma unroll
        for (int t = 0; t < MT; ++t)
#pragma unroll
          for (int u = 0; u < NT; ++u) red[((wave - 1) * MT * NT + t * NT + u) * 64 + lane] = acc[t][u];
      }
      __syncthreads();
      if (wave == 0) {
#pragma unroll
        for (int w = 0; w < 3; ++w)
#pragma unroll
          for (int t = 0; t < MT; ++t)
#pragma unroll
            for (int u = 0; u < NT; ++u) {
              f32x4 v = red[(w * MT * NT + t * NT + u) * 64 + lane];
              acc[t][u] += v;
            }
      }
      active = active && wave == 0;
    }
  }
  // after run(): for the owning wave, acc[t][u][r] is the value for
  //   row  m = m0 + 16 t + lane%16,  column n = 16 (nt0+u) + 4 (lane/16) + r.
};

template <int MT, int NT, int KS>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(GemmP p, Epi e) {
  __shared__ f32x4 red[KS == 4 ? 3 * MT * NT * 64 : 1];
  GemmMain<MT, NT, KS> g;
  g.run(p, red);
  if (!g.active) return;
  const int ntiles = p.N >> 4;
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int m = g.m0 + t * 16 + (g.lane & 15);
    if (m >= p.M) continue;
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      if (g.nt0 + u >= ntiles) continue;
      const int n = (g.nt0 + u) * 16 + (g.lane >> 4) * 4;
#pragma unroll
      for (int r = 0; r < 4; ++r) epi_store<bf16_t>(e, blockIdx.z, m, n + r, g.acc[t][u][r]);
    }
  }
}

// Order-preserving map float -> uint32, then (value, lowest index wins) packed in 64 bits so
// that an unsigned max over keys is the argmax regardless of the order of the updates.
__device__ __forceinline__ unsigned long long argmax_key(float v, unsigned idx) {
  unsigned u = __float_as_uint(v);
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((unsigned long long)u << 32) | (unsigned long long)(0xFFFFFFFFu - idx);
}
__device__ __forceinline__ int key_index(unsigned long long key) {
  return (int)(0xFFFFFFFFu - (unsigned)(key & 0xFFFFFFFFull));
}

// Vocabulary projection with the arg-max over the vocabulary fused into the epilogue: the
// logits of the k x k outputs per sequence are never written unless `logits` is given.
template <int MT, int NT, int KS>
__global__ __launch_bounds__(256) void vocab_argmax_bf16_kernel(GemmP p, unsigned long long* keys,
                                                                float* logits) {
  __shared__ f32x4 red[KS == 4 ? 3 * MT * NT * 64 : 1];
  GemmMain<MT, NT, KS> g;
  g.run(p, red);
  if (!g.active) return;
  const int ntiles = p.N >> 4;
#pragma unroll
  for (int t = 0; t < MT; ++t) {
    const int m = g.m0 + t * 16 + (g.lane & 15);
    unsigned long long best = 0ull;
#pragma unroll
    for (int u = 0; u < NT; ++u) {
      if (g.nt0 + u >= ntiles) continue;
      const int n = (g.nt0 + u) * 16 + (g.lane >> 4) * 4;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float v = g.acc[t][u][r];
        const unsigned long long key = argmax_key(v, (unsigned)(n + r));
        best = key > best ? key : best;
        if (logits && m < p.M) logits[(long)m * p.N + n + r] = v;
      }
    }
    // lanes l, l^16, l^32, l^48 hold the same row
    unsigned long long o = __shfl_xor(best, 16, 64); best = o > best ? o : best;
    o = __shfl_xor(best, 32, 64); best = o > best ? o : best;
    if (g.lane < 16 && m < p.M) atomicMax(&keys[m], best);
  }
}

#include "bpd_gemm.h"

// ---------------------------------------------------------------------------------------
// fp32 mode (small configurations): one thread per output element.
__global__ void gemm_f32_kernel(GemmP p, Epi e) {
  const int n = blockIdx.x * blockDim.x + threadIdx.x;
  const int m = blockIdx.y, g = blockIdx.z;
  if (n >= p.N || m >= p.M) return;
  const float* X = (const float*)p.X + g * p.x_g + (long)m * p.ldx;
  const float* W = (const float*)p.W + g * p.w_g + n;
  float acc = 0.f;
  int k = 0;
  for (; k + 8 <= p.K; k += 8) {               // eight loads in flight, then the same sequential sum as the tail loop
    float xv[8], wv[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) { xv[j] = X[k + j]; wv[j] = W[(long)(k + j) * p.ldw]; }
#pragma unroll
    for (int j = 0; j < 8; ++j) acc = fmaf(xv[j], wv[j], acc);
  }
  for (; k < p.K; ++k) acc = fmaf(X[k], W[(long)k * p.ldw], acc);
  epi_store<float>(e, g, m, n, acc);
}

// fp32 vocabulary projection: E is [V][d] row-major; one workgroup per row of O.
__global__ __launch_bounds__(256) void vocab_argmax_f32_kernel(const float* O, int ldo, const float* E, int M, int V,
                                                               int d, unsigned long long* keys, float* logits) {
  const int m = blockIdx.x;
  if (m >= M) return;
  const float* o = O + (long)m * ldo;
  unsigned long long best = 0ull;
  for (int v = threadIdx.x; v < V; v += blockDim.x) {
    const float* ev = E + (long)v * d;
    float acc = 0.f;
    int c = 0;
    for (; c + 8 <= d; c += 8) {
      float ov[8], wv[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) { ov[j] = o[c + j]; wv[j] = ev[c + j]; }
#pragma unroll
      for (int j = 0; j < 8; ++j) acc = fmaf(ov[j], wv[j], acc);
    }
    for (; c < d; ++c) acc = fmaf(o[c], ev[c], acc);
    if (logits) logits[(long)m * V + v] = acc;
    const unsigned long long key = argmax_key(acc, (unsigned)v);
    best = key > best ? key : best;
  }
  for (int off = 32; off > 0; off >>= 1) {
    unsigned long long o2 = __shfl_xor(best, off, 64);
    best = o2 > best ? o2 : best;
  }
  if ((threadIdx.x & 63) == 0) atomicMax(&keys[m], best);
}

// ---------------------------------------------------------------------------------------
// Weight conversion at load time.
// src: [K][N_src] row-major (or, transposed, [N_src][K]) of float or bf16 bits.
// bf16 mode: dst = packed tiles of a matrix with K rows; the tensor lands at columns n_off..
// fp32 mode: dst = row-major [K][ldw] fp32, columns n_off..
template <typename SRC, bool PACK>
__global__ void convert_matrix_kernel(const SRC* src, void* dst, int K, int Nsrc, int transposed,
                                      int ldw, int n_off) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx >= (long)K * Nsrc) return;
  int k, n;
  if (transposed) { n = (int)(idx / K); k = (int)(idx % K); } else { k = (int)(idx / Nsrc); n = (int)(idx % Nsrc); }
  const float v = to_f<SRC>(src[idx]);
  const int nn = n + n_off;
  if (PACK) {
    const int ksteps = K >> 5;
    const long tile = (long)(nn >> 4) * ksteps + (k >> 5);
    const int lane = 16 * ((k & 31) >> 3) + (nn & 15);
    ((bf16_t*)dst)[(tile * 64 + lane) * 8 + (k & 7)] = f2bf(v);
  } else {
    ((float*)dst)[(long)k * ldw + nn] = v;
  }
}

template <typename SRC>
__global__ void convert_vector_kernel(const SRC* src, float* dst, long n) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < n) dst[idx] = to_f<SRC>(src[idx]);
}

// LayerNorm folded into the weights that follow it: LN(x) W = rstd * (x W' - mu * c) + dvec with
//   W'[k][n] = g[k] W[k][n] (rounded to bf16),  c[n] = sum_k W'[k][n] (of the rounded values: what the matrix cores
//   multiply),  dvec[n] = sum_k b[k] W[k][n].
// Wp / Wf: packed tiles [N/16][K/32][64 lanes][8]; one wavefront per column tile.  Grid N/16, 64 threads.
__global__ __launch_bounds__(64) void fold_layernorm_kernel(const bf16_t* Wp, bf16_t* Wf, const float* g, const float* b,
                                                            float* c, float* dvec, int ksteps) {
  const int tile = blockIdx.x, lane = threadIdx.x;
  float cs = 0.f, ds = 0.f;
  for (int ks = 0; ks < ksteps; ++ks) {
    const long at = (((long)tile * ksteps + ks) * 64 + lane) * 8;
    const uint4 raw = *(const uint4*)(Wp + at);
    const unsigned in[4] = {raw.x, raw.y, raw.z, raw.w};
    unsigned out[4];
    const int k0 = ks * 32 + (lane >> 4) * 8;
#pragma unroll
    for (int e2 = 0; e2 < 4; ++e2) {
      const float w0 = __uint_as_float(in[e2] << 16), w1 = __uint_as_float(in[e2] & 0xFFFF0000u);
      const bf16_t f0 = f2bf(w0 * g[k0 + 2 * e2]), f1 = f2bf(w1 * g[k0 + 2 * e2 + 1]);
      cs += bf2f(f0) + bf2f(f1);
      ds = fmaf(b[k0 + 2 * e2], w0, ds); ds = fmaf(b[k0 + 2 * e2 + 1], w1, ds);
      out[e2] = (unsigned)f0 | ((unsigned)f1 << 16);
    }
    *(uint4*)(Wf + at) = make_uint4(out[0], out[1], out[2], out[3]);
  }
  cs += __shfl_xor(cs, 16, 64); cs += __shfl_xor(cs, 32, 64);
  ds += __shfl_xor(ds, 16, 64); ds += __shfl_xor(ds, 32, 64);
  if (lane < 16) { c[tile * 16 + lane] = cs; dvec[tile * 16 + lane] = ds; }
}

// ---------------------------------------------------------------------------------------
// Embedding of the k proposed tokens (decoder side) or of the source tokens.
//   x[row][c] = sqrt(d) * E[tok][c] + pos[position][c];  tok < 0 -> zero vector (the shifted
//   decoder input at position 0).  E is the packed vocabulary matrix in bf16 mode.
template <bool BF16>
__global__ void embed_kernel(const int* tok, int tok_ld, const int* base, int rows_per_seq, int M,
                             int d, const void* E, int V, const float* pos, float scale, float* x,
                             int zero_input, unsigned long long* keys, int nkeys) {
  const long idx = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (idx < nkeys) keys[idx] = 0ull;          // argmax keys of this invocation start at "nothing"
  if (idx >= (long)M * d) return;
  const int row = (int)(idx / d), c = (int)(idx % d);
  const int b = row / rows_per_seq, i = row % rows_per_seq;
  const int position = (base ? base[b] : 0) + i;
  float v = pos[(long)position * d + c];
  if (!zero_input) {
    int t = tok[b * tok_ld + i];
    t = t < 0 ? 0 : (t >= V ? V - 1 : t);      // ids are validated on the host; never index outside E
    float ev;
    if (BF16) {
      const int ksteps = d >> 5;
      const long tile = (long)(t >> 4) * ksteps + (c >> 5);
      const int lane = 16 * ((c & 31) >> 3) + (t & 15);
      ev = bf2f(((const bf16_t*)E)[(tile * 64 + lane) * 8 + (c & 7)]);
    } else {
      ev = ((const float*)E)[(long)t * d + c];
    }
    v += scale * ev;
  }
  x[idx] = v;
}

// Embedding for a block of <= 16 rows (bf16 mode): one wavefront per 16-column tile, lane =
// (row = lane % 16, 4 columns), so that the tile's partial LayerNorm statistics (sum, sum of
// squares per row) are written along with x, in the layout row_stats() reads.
__global__ __launch_bounds__(64) void embed_stats_kernel(const int* tok, int tok_ld, const int* base, int rows_per_seq,
                                                         int M, int d, const bf16_t* E, int V, const float* pos,
                                                         float scale, float* x, int zero_input, float* stats,
                                                         unsigned long long* keys, int nkeys) {
  const int tile = blockIdx.x, lane = threadIdx.x;
  for (int i = tile * 64 + lane; i < nkeys; i += gridDim.x * 64) keys[i] = 0ull;
  const int row = lane & 15, c0 = tile * 16 + (lane >> 4) * 4;
  const int r = row < M ? row : M - 1;
  const int b = r / rows_per_seq, i = r % rows_per_seq;
  const int position = (base ? base[b] : 0) + i;
  const float4 pv = *(const float4*)(pos + (long)position * d + c0);
  float v[4] = {pv.x, pv.y, pv.z, pv.w};
  if (!zero_input) {
    int t = tok[b * tok_ld + i];
    t = t < 0 ? 0 : (t >= V ? V - 1 : t);
    const int ksteps = d >> 5;
    const long tl = (long)(t >> 4) * ksteps + (c0 >> 5);
    const int ln = 16 * ((c0 & 31) >> 3) + (t & 15);
    const uint2 raw = *(const uint2*)(E + (tl * 64 + ln) * 8 + (c0 & 7));
    v[0] += scale * __uint_as_float(raw.x << 16); v[1] += scale * __uint_as_float(raw.x & 0xFFFF0000u);
    v[2] += scale * __uint_as_float(raw.y << 16); v[3] += scale * __uint_as_float(raw.y & 0xFFFF0000u);
  }
  float s = (v[0] + v[1]) + (v[2] + v[3]);
  float q = (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
  s += __shfl_xor(s, 16, 64); s += __shfl_xor(s, 32, 64);
  q += __shfl_xor(q, 16, 64); q += __shfl_xor(q, 32, 64);
  if (lane < 16) ((float2*)stats)[tile * 16 + lane] = make_float2(s, q);
  if (row < M) *(float4*)(x + (long)row * d + c0) = make_float4(v[0], v[1], v[2], v[3]);
}

// LayerNorm over the last axis, one wavefront per row (biased variance, two passes over
// registers).  The row is fetched with one batch of loads; d <= 64 * 4 * LN_V.
// If the producer of x was a split-K GEMM (nsl > 0 slices of the product in `part`, slice s at
// part + s*M*d), the row is first completed, x += bias + part[0] + part[1] + ... in that order,
// and written back.
constexpr int LN_V = 8;
template <typename ACT, int V>
__global__ __launch_bounds__(256) void layernorm_kernel(float* x, const float* g, const float* b, int M,
                                                        int d, float eps, ACT* ya, float* yf,
                                                        const float* part, int nsl, const float* pbias) {
  const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  if (row >= M) return;
  float* xr = x + (long)row * d;
  const int nv = d >> 2;                         // float4 per row
  float4 v[V], gg[V], bb[V];
#pragma unroll
  for (int i = 0; i < V; ++i) {
    const int c4 = lane + 64 * i;
    const int cc = c4 < nv ? c4 : 0;
    v[i] = ((const float4*)xr)[cc]; gg[i] = ((const float4*)g)[cc]; bb[i] = ((const float4*)b)[cc];
  }
  if (nsl > 0) {
    float4 pb[V];
#pragma unroll
    for (int i = 0; i < V; ++i) {
      const int c4 = lane + 64 * i;
      pb[i] = ((const float4*)pbias)[c4 < nv ? c4 : 0];
    }
    // four slices per batch of loads; the first batch is requested together with the row, gain / bias and the slices'
    // bias (one round trip), the additions keep their order: x + bias + part[0] + part[1] + ...
    float4 q[4][V];
#define BPD_LN_LOAD_SLICES(s0)                                                                  \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                             \
      const int sl = (s0) + j < nsl ? (s0) + j : nsl - 1;                                       \
      const float4* pr = (const float4*)(part + ((long)sl * M + row) * d);                      \
      _Pragma("unroll") for (int i = 0; i < V; ++i) {                                           \
        const int c4 = lane + 64 * i;                                                           \
        q[j][i] = pr[c4 < nv ? c4 : 0];                                                         \
      }                                                                                         \
    }
#define BPD_LN_ADD_SLICES(s0)                                                                   \
    _Pragma("unroll") for (int j = 0; j < 4; ++j) {                                             \
      const float w = (s0) + j < nsl ? 1.f : 0.f;                                               \
      _Pragma("unroll") for (int i = 0; i < V; ++i) {                                           \
        v[i].x = fmaf(w, q[j][i].x, v[i].x); v[i].y = fmaf(w, q[j][i].y, v[i].y);               \
        v[i].z = fmaf(w, q[j][i].z, v[i].z); v[i].w = fmaf(w, q[j][i].w, v[i].w);               \
      }                                                                                         \
    }
    BPD_LN_LOAD_SLICES(0)
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < V; ++i) { v[i].x += pb[i].x; v[i].y += pb[i].y; v[i].z += pb[i].z; v[i].w += pb[i].w; }
    BPD_LN_ADD_SLICES(0)
    for (int s0 = 4; s0 < nsl; s0 += 4) {
      BPD_LN_LOAD_SLICES(s0)
      BPD_LN_ADD_SLICES(s0)
    }
#undef BPD_LN_ADD_SLICES
#undef BPD_LN_LOAD_SLICES
#pragma unroll
    for (int i = 0; i < V; ++i) {
      const int c4 = lane + 64 * i;
      if (c4 < nv) ((float4*)xr)[c4] = v[i];
    }
  }
  __builtin_amdgcn_sched_barrier(0);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < V; ++i) {
    const float w = (lane + 64 * i) < nv ? 1.f : 0.f;
    s += w * ((v[i].x + v[i].y) + (v[i].z + v[i].w));
  }
  const float mu = wave_sum(s) / d;
  float q = 0.f;
#pragma unroll
  for (int i = 0; i < V; ++i) {
    const float w = (lane + 64 * i) < nv ? 1.f : 0.f;
    const float a0 = v[i].x - mu, a1 = v[i].y - mu, a2 = v[i].z - mu, a3 = v[i].w - mu;
    q += w * ((a0 * a0 + a1 * a1) + (a2 * a2 + a3 * a3));
  }
  const float rstd = 1.0f / sqrtf(wave_sum(q) / d + eps);
#pragma unroll
  for (int i = 0; i < V; ++i) {
    const int c4 = lane + 64 * i;
    if (c4 < nv) {
      const float y0 = (v[i].x - mu) * rstd * gg[i].x + bb[i].x, y1 = (v[i].y - mu) * rstd * gg[i].y + bb[i].y;
      const float y2 = (v[i].z - mu) * rstd * gg[i].z + bb[i].z, y3 = (v[i].w - mu) * rstd * gg[i].w + bb[i].w;
      if (ya) {
        ACT* o = ya + (long)row * d + 4 * c4;
        if constexpr (sizeof(ACT) == 2) {          // bf16: one 8-byte store
          *(uint2*)o = make_uint2((unsigned)f2bf(y0) | ((unsigned)f2bf(y1) << 16), (unsigned)f2bf(y2) | ((unsigned)f2bf(y3) << 16));
        } else {
          o[0] = from_f<ACT>(y0); o[1] = from_f<ACT>(y1); o[2] = from_f<ACT>(y2); o[3] = from_f<ACT>(y3);
        }
      }
      if (yf) ((float4*)(yf + (long)row * d))[c4] = make_float4(y0, y1, y2, y3);
    }
  }
}

// ---------------------------------------------------------------------------------------
// Attention of a tile of <= 16 query rows of one (sequence, head) over keys 0..n-1 held in a
// K/V buffer: the decoder self-attention over the cache plus the block (block-causal: row i
// sees keys < base[b] + i + 1), the cross attention (keys < len[b]) and the encoder's
// self-attention.  Keys are visited in chunks of 256 with a running (max, sum) per row so
// the LDS footprint does not depend on the cache length.
//   Q    fp32 [B*R][d]                 out  act [B*R][d]
//   Kc,Vc act, sequence b at Kc + b*kv_seq_stride, key s at + s*d, head h at + h*DH
template <typename ACT, int DH> struct RowLoader;
template <int DH> struct RowLoader<float, DH> {
  static __device__ __forceinline__ void unpack(const uint4* raw, float* out) {
#pragma unroll
    for (int x = 0; x < DH / 4; ++x) {
      out[4 * x] = __uint_as_float(raw[x].x); out[4 * x + 1] = __uint_as_float(raw[x].y);
      out[4 * x + 2] = __uint_as_float(raw[x].z); out[4 * x + 3] = __uint_as_float(raw[x].w);
    }
  }
  static __device__ __forceinline__ void load(const float* p, float* out) {
#pragma unroll
    for (int x = 0; x < DH; x += 4) {
      const float4 v = *(const float4*)(p + x);
      out[x] = v.x; out[x + 1] = v.y; out[x + 2] = v.z; out[x + 3] = v.w;
    }
  }
};
template <int DH> struct RowLoader<bf16_t, DH> {
  static __device__ __forceinline__ void unpack(const uint4* raw, float* out) {
#pragma unroll
    for (int x = 0; x < DH / 8; ++x) {
      const unsigned w[4] = {raw[x].x, raw[x].y, raw[x].z, raw[x].w};
#pragma unroll
      for (int y = 0; y < 4; ++y) {
        out[8 * x + 2 * y] = __uint_as_float(w[y] << 16);
        out[8 * x + 2 * y + 1] = __uint_as_float(w[y] & 0xFFFF0000u);
      }
    }
  }
  static __device__ __forceinline__ void load(const bf16_t* p, float* out) {
#pragma unroll
    for (int x = 0; x < DH; x += 8) {
      const uint4 v = *(const uint4*)(p + x);
      const unsigned w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
      for (int y = 0; y < 4; ++y) {
        out[x + 2 * y] = __uint_as_float(w[y] << 16);
        out[x + 2 * y + 1] = __uint_as_float(w[y] & 0xFFFF0000u);
      }
    }
  }
};

struct AttnP {
  const float* Q;
  const void* Kc; const void* Vc;
  void* out;
  long kv_seq_stride;
  int cap;                // rows per sequence in the K/V buffer (loads are clamped to it)
  int d, R;
  const int* limit;       // [B]: base (causal) or len (non-causal)
  int causal;
  float scale;
  int local_q, local_m;   // causal only, local_q > 0: 1D local attention (Section 7.2): the row at position t sees keys
                          // floor(t / local_q) * local_q - local_m .. t; the chunks then start at the first row's bound
  int nsplit;             // key chunks are dealt round-robin to nsplit workgroups per (head, sequence, row tile)
  float* part;            // nsplit > 1: partial results [b][h][tile][split][16*DH acc | 16 max | 16 sum]
};

// first key that the row at position t may see
__device__ __forceinline__ int attn_first_key(const AttnP& p, int t) {
  if (!(p.causal && p.local_q > 0)) return 0;
  const int lo = t / p.local_q * p.local_q - p.local_m;
  return lo > 0 ? lo : 0;
}

// With nsplit == 1 the kernel writes the attention output.  With nsplit > 1 (long caches, few
// sequences) every workgroup leaves its running maximum, sum and un-normalised weighted values
// in p.part and attention_combine_kernel merges them.
template <typename ACT, int DH>
__global__ __launch_bounds__(256) void attention_kernel(AttnP p) {
  constexpr int RT = 16, CH = 256, G = 256 / DH, KPG = CH / G, SLD = CH + 4;
  __shared__ __attribute__((aligned(16))) float q_s[RT][DH];
  __shared__ __attribute__((aligned(16))) float sc[RT][SLD];
  __shared__ __attribute__((aligned(16))) ACT vs[CH][DH];
  __shared__ float m_s[RT], l_s[RT], alpha_s[RT];
  const int h = blockIdx.x, b = blockIdx.y;
  const int split = blockIdx.z % p.nsplit, tile = blockIdx.z / p.nsplit, r0 = tile * RT;
  int kbeg = 0;                                  // local attention: the length decides where the keys start (read first)
  if (p.causal && p.local_q > 0) { const int l0 = p.limit[b]; kbeg = attn_first_key(p, (l0 < 0 ? 0 : l0) + r0); }
  const int first = kbeg + split * CH, hop = p.nsplit * CH;
  const int nrows = min(RT, p.R - r0);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const ACT* Kb = (const ACT*)p.Kc + b * p.kv_seq_stride + h * DH;
  const ACT* Vb = (const ACT*)p.Vc + b * p.kv_seq_stride + h * DH;
  // first chunk's K and V rows are requested before anything else: one memory round trip
  constexpr int VW = DH * sizeof(ACT) / 16;               // 16-byte words per row
  uint4 kraw[VW], vraw[VW];
  {
    const int key = first + tid < p.cap ? first + tid : p.cap - 1;   // independent of the length: no second round trip
    const uint4* kp = (const uint4*)(Kb + (long)key * p.d);
    const uint4* vp = (const uint4*)(Vb + (long)key * p.d);
#pragma unroll
    for (int x = 0; x < VW; ++x) { kraw[x] = kp[x]; vraw[x] = vp[x]; }
  }
  // queries: RT*DH/256 consecutive features per thread, one unconditional load (rows clamped)
  constexpr int QE = RT * DH / 256;
  float qreg[QE];
  {
    const int i = tid * QE / DH, c = tid * QE % DH;
    const int row = r0 + (i < nrows ? i : nrows - 1);
    const float* qp = p.Q + ((long)b * p.R + row) * p.d + h * DH + c;
    if (QE == 4) { const float4 v = *(const float4*)qp; qreg[0] = v.x; qreg[1 % QE] = v.y; qreg[2 % QE] = v.z; qreg[3 % QE] = v.w; }
    else {
#pragma unroll
      for (int x = 0; x < QE; ++x) qreg[x] = qp[x];
    }
  }
  int lim = p.limit[b];
  lim = lim < 0 ? 0 : lim;
  int nkeys = p.causal ? lim + r0 + nrows : lim;   // keys any row of the tile can see
  nkeys = nkeys < p.cap ? nkeys : p.cap;
  __builtin_amdgcn_sched_barrier(0);              // all global loads above are in flight before the first wait
  {
    const int i = tid * QE / DH, c = tid * QE % DH;
#pragma unroll
    for (int x = 0; x < QE; ++x) q_s[i][c + x] = i < nrows ? qreg[x] * p.scale : 0.f;
  }
  if (tid < RT) { m_s[tid] = -INFINITY; l_s[tid] = 0.f; alpha_s[tid] = 1.f; }
  float acc[RT];
#pragma unroll
  for (int i = 0; i < RT; ++i) acc[i] = 0.f;
  const int g = tid / DH, c = tid % DH;
  __syncthreads();
  for (int c0 = first; c0 < nkeys; c0 += hop) {
    const int key = c0 + tid;
    if (c0 != first) {
      const int kk = key < nkeys ? key : 0;
      const uint4* kp = (const uint4*)(Kb + (long)kk * p.d);
      const uint4* vp = (const uint4*)(Vb + (long)kk * p.d);
#pragma unroll
      for (int x = 0; x < VW; ++x) { kraw[x] = kp[x]; vraw[x] = vp[x]; }
    }
    // scores of this chunk: one key per thread
    {
      float kr[DH];
      RowLoader<ACT, DH>::unpack(kraw, kr);
      for (int i = 0; i < nrows; ++i) {
        float s = 0.f;
#pragma unroll
        for (int x = 0; x < DH; x += 4) {
          const float4 qv = *(const float4*)&q_s[i][x];
          s = fmaf(qv.x, kr[x], s); s = fmaf(qv.y, kr[x + 1], s);
          s = fmaf(qv.z, kr[x + 2], s); s = fmaf(qv.w, kr[x + 3], s);
        }
        const int nvis = p.causal ? lim + r0 + i + 1 : lim;
        sc[i][tid] = (key < nvis && key >= attn_first_key(p, lim + r0 + i)) ? s : -INFINITY;
      }
      const bool live = key < nkeys;
#pragma unroll
      for (int x = 0; x < VW; ++x) ((uint4*)&vs[tid][0])[x] = live ? vraw[x] : make_uint4(0, 0, 0, 0);
    }
    __syncthreads();
    // running max / sum: 16 lanes per row, 4 rows per wave at once
    {
      const int i = wave * 4 + (lane >> 4), j0 = lane & 15;
      if (i < nrows) {
        float v[16], mx = -INFINITY;
#pragma unroll
        for (int x = 0; x < 16; ++x) { v[x] = sc[i][j0 + 16 * x]; mx = fmaxf(mx, v[x]); }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) mx = fmaxf(mx, __shfl_xor(mx, o, 64));
        const float m_old = m_s[i];
        const float m_new = fmaxf(m_old, mx);
        float sum = 0.f;
#pragma unroll
        for (int x = 0; x < 16; ++x) {
          const float pv = (m_new == -INFINITY) ? 0.f : __expf(v[x] - m_new);
          sc[i][j0 + 16 * x] = pv;
          sum += pv;
        }
#pragma unroll
        for (int o = 8; o > 0; o >>= 1) sum += __shfl_xor(sum, o, 64);
        if (j0 == 0) {
          const float a = (m_new == -INFINITY) ? 1.f : __expf(m_old - m_new);
          alpha_s[i] = a;
          l_s[i] = l_s[i] * a + sum;
          m_s[i] = m_new;
        }
      } else if (i < RT) {
#pragma unroll
        for (int x = 0; x < 16; ++x) sc[i][j0 + 16 * x] = 0.f;      // unused rows contribute nothing
      }
    }
    __syncthreads();
    // weighted values: thread (g, c) takes keys g*KPG .. of the chunk for feature c
#pragma unroll
    for (int i = 0; i < RT; ++i) acc[i] *= alpha_s[i];
    const int kend = min(CH, nkeys - c0);
    for (int kk = g * KPG; kk < min((g + 1) * KPG, kend); kk += 4) {
      float vv[4];
#pragma unroll
      for (int y = 0; y < 4; ++y) vv[y] = to_f<ACT>(vs[kk + y][c]);
#pragma unroll
      for (int i = 0; i < RT; ++i) {
        const float4 pv = *(const float4*)&sc[i][kk];
        acc[i] = fmaf(pv.x, vv[0], acc[i]); acc[i] = fmaf(pv.y, vv[1], acc[i]);
        acc[i] = fmaf(pv.z, vv[2], acc[i]); acc[i] = fmaf(pv.w, vv[3], acc[i]);
      }
    }
    __syncthreads();
  }
  // sum over the G key groups (reusing the score buffer), normalise, write
  float* red = &sc[0][0];                     // needs G*RT*DH = 4096 floats <= RT*SLD
#pragma unroll
  for (int i = 0; i < RT; ++i) red[(g * RT + i) * DH + c] = acc[i];
  __syncthreads();
  if (p.nsplit == 1) {
    for (int idx = tid; idx < nrows * DH; idx += 256) {
      const int i = idx / DH, cc = idx % DH;
      float s = 0.f;
      for (int gg = 0; gg < G; ++gg) s += red[(gg * RT + i) * DH + cc];
      ((ACT*)p.out)[((long)b * p.R + r0 + i) * p.d + h * DH + cc] = from_f<ACT>(s / l_s[i]);
    }
  } else {
    const int tiles = gridDim.z / p.nsplit;
    float* part = p.part + ((((long)b * gridDim.x + h) * tiles + tile) * p.nsplit + split) * (RT * (DH + 2));
    for (int idx = tid; idx < RT * DH; idx += 256) {
      const int i = idx / DH, cc = idx % DH;
      float s = 0.f;
      for (int gg = 0; gg < G; ++gg) s += red[(gg * RT + i) * DH + cc];
      part[idx] = s;
    }
    if (tid < RT) { part[RT * DH + tid] = m_s[tid]; part[RT * DH + RT + tid] = l_s[tid]; }
  }
}

// bf16, 64-wide heads: the same computation on the matrix cores, one barrier per workgroup.  The four waves split
// the keys: of every 256-key chunk wave w takes keys 64w .. 64w+63 and keeps its own running maximum, sum and weighted
// values in registers; the waves' results meet once, in LDS, at the end.  Per chunk and wave
//   scores^T = K Q^T     keys are the 16-wide "feature" side of the MFMA, the <= 16 query rows the other; K fragments
//                        come straight from the cache (a key row is contiguous along the contracted head dimension);
//                        a lane then holds, for its query row, the scores of 4 keys of each of the 4 key tiles
//   softmax              maximum and sum over the wave's 64 keys: in the lane, then across the 4 lanes of a row;
//                        the probabilities stay in registers: the scores of two key tiles are, as they lie, the
//                        second MFMA operand for a contraction over those 32 keys (in a permuted key order)
//   out^T += V^T P^T     contracted over keys, 64 head dimensions = 4 output tiles; the V^T fragments (same key
//                        order) are gathered from the wave's own 64 V rows staged in LDS (row stride 68 elements,
//                        so the four key groups of a fragment read disjoint banks; no barrier: a wave's LDS
//                        accesses execute in order)
// fp32 operands (Q, the probabilities) are fed as a bf16 pair hi + lo, which keeps them to ~2^-17: the result matches
// the scalar kernel to fp32 rounding.  Same arguments, grid and partial-result layout as attention_kernel.
__device__ __forceinline__ void split_bf16x8(const float (&v)[8], bf16x8& hi, bf16x8& lo) {
  unsigned h[4], l[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const bf16_t h0 = f2bf(v[2 * j]), h1 = f2bf(v[2 * j + 1]);
    const bf16_t l0 = f2bf(v[2 * j] - bf2f(h0)), l1 = f2bf(v[2 * j + 1] - bf2f(h1));
    h[j] = (unsigned)h0 | ((unsigned)h1 << 16);
    l[j] = (unsigned)l0 | ((unsigned)l1 << 16);
  }
  hi = __builtin_bit_cast(bf16x8, make_uint4(h[0], h[1], h[2], h[3]));
  lo = __builtin_bit_cast(bf16x8, make_uint4(l[0], l[1], l[2], l[3]));
}

__device__ __forceinline__ unsigned pack_bf16_pair(float lo, float hi) { return (unsigned)f2bf(lo) | ((unsigned)f2bf(hi) << 16); }

// KVNT: K and V are fetched with non-temporal loads (a cache too large for the last-level cache is a
// stream that should not evict the weights).
typedef unsigned int u32x4_kv __attribute__((ext_vector_type(4)));
// LIMF: the sequence's length is fetched first and the K/V loads are clamped to it instead of to the buffer's rows: one
// more dependent round trip, but rows past the end are not fetched (many sequences: the traffic is what counts).
// QU > 0 (at most 16 rows per sequence, d = 128 * QU): the queries are projected inside the kernel,
//   Q = LayerNorm(x) Wq[:, 64 h .. 64 h + 63]   (x: fp32 residual stream with its partial LayerNorm statistics),
// instead of being read from p.Q: the four waves split the contraction, their partial sums meet in LDS, and the K/V
// loads of the first chunk are already in flight meanwhile.  Saves the projection's kernel and its round trip.
struct QProjP {
  const float* x;       // [M][d] residual stream
  const float* g;       // LayerNorm gain, bias
  const float* b;
  const float* stats;   // partial statistics of x: [(part * srows + row) * 2]
  int srows;            // 16: single-tile path, one part per 16 columns; otherwise M rows, one part per 64 columns
  const void* W;        // packed [d/16 column tiles][d/32 k-steps][64 lanes][8]
  float eps;
};
// LDS of one attention workgroup (4 waves): the kernel below declares it; a caller that runs the body from inside
// another kernel carves it out of its own LDS.
struct AttnLds {
  static constexpr int RT = 16, DH = 64, WK = 64, VLD = DH + 4;
  bf16_t (*vs)[WK][VLD];      // [4][WK][VLD] per wave: its 64 V rows of the chunk
  f32x4 (*o_s)[4][64];        // [4][4][64]   per wave and output tile: un-normalised out^T
  float (*m_s)[RT];           // [4][RT]      per wave: running maximum per query row
  float (*l_s)[RT];           // [4][RT]      ... and sum
  float* q_s;                 // QU > 0: [RT * (DH + 4)] projected queries
  static constexpr size_t VS_BYTES = (size_t)4 * WK * VLD * 2, OS_BYTES = (size_t)4 * 4 * 64 * 16, ML_BYTES = (size_t)4 * RT * 4;
  static constexpr size_t BYTES = VS_BYTES + OS_BYTES + 2 * ML_BYTES;        // without q_s
  // carve (16-byte aligned base), QU == 0 layout
  __device__ static AttnLds carve(unsigned char* base) {
    AttnLds s;
    s.vs = (bf16_t (*)[WK][VLD])base;
    s.o_s = (f32x4 (*)[4][64])(base + VS_BYTES);
    s.m_s = (float (*)[RT])(base + VS_BYTES + OS_BYTES);
    s.l_s = (float (*)[RT])(base + VS_BYTES + OS_BYTES + ML_BYTES);
    s.q_s = nullptr;
    return s;
  }
};
// One (head h, sequence b, z = row tile * nsplit + split) item of the attention, run by 256 threads (tid 0..255, four
// whole waves) that share `sm`; nheads / nz: the extents the partial-result layout is indexed with.  Every
// __syncthreads() inside is reached by all 256 threads; a caller whose workgroup has more waves makes those arrive at
// as many barriers (one with QU == 0, three with QU > 0).
template <bool KVNT, bool LIMF, int QU>
__device__ __forceinline__ void attention_mfma_body(const AttnP& p, const QProjP& qp, const AttnLds& sm, int h, int b, int z,
                                                    int nheads, int nz, int tid) {
  constexpr int RT = 16, CH = 256, DH = 64, WK = 64, VLD = DH + 4;
  bf16_t (*vs)[WK][VLD] = sm.vs;
  f32x4 (*o_s)[4][64] = sm.o_s;
  float (*m_s)[RT] = sm.m_s;
  float (*l_s)[RT] = sm.l_s;
  float* q_s = sm.q_s;
  const int split = z % p.nsplit, tile = z / p.nsplit, r0 = tile * RT;
  const int nrows = min(RT, p.R - r0);
  const int lane = tid & 63, wave = tid >> 6;
  const int lr = lane & 15, lq = lane >> 4;
  const bf16_t* Kb = (const bf16_t*)p.Kc + b * p.kv_seq_stride + h * DH;
  const bf16_t* Vb = (const bf16_t*)p.Vc + b * p.kv_seq_stride + h * DH;
  int kmax = p.cap;                              // rows that may be fetched
  int kbeg = 0;                                  // first key of the first chunk (local attention: LIMF only)
  if (LIMF) {
    int l0 = p.limit[b];
    l0 = l0 < 0 ? 0 : l0;
    const int nk0 = p.causal ? l0 + r0 + nrows : l0;
    kmax = nk0 < p.cap ? (nk0 > 0 ? nk0 : 1) : p.cap;
    kbeg = attn_first_key(p, l0 + r0);
  }
  const int first = kbeg + split * CH, hop = p.nsplit * CH;
  // K fragments (4 key tiles x 2 halves of the head dimension) and this lane's 8 pieces of the wave's V rows
  uint4 kf[4][2], vraw[8];
#define BPD_LOAD_KV(c0)                                                                         \
  {                                                                                             \
    _Pragma("unroll") for (int kt = 0; kt < 4; ++kt) {                                          \
      int key = (c0) + wave * WK + kt * 16 + lr;                                                \
      key = key < kmax ? key : kmax - 1;                                                        \
      const bf16_t* kp = Kb + (long)key * p.d + 8 * lq;                                         \
      if (KVNT) {                                                                               \
        kf[kt][0] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_kv*)kp));     \
        kf[kt][1] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_kv*)(kp + 32))); \
      } else {                                                                                  \
        kf[kt][0] = *(const uint4*)kp; kf[kt][1] = *(const uint4*)(kp + 32);                    \
      }                                                                                         \
    }                                                                                           \
    _Pragma("unroll") for (int x = 0; x < 8; ++x) {       /* 8 lanes per V row: a wave-load covers 8 whole rows */ \
      int vkey = (c0) + wave * WK + 8 * x + (lane >> 3);                                        \
      vkey = vkey < kmax ? vkey : kmax - 1;                                                     \
      const bf16_t* vp_ = Vb + (long)vkey * p.d + 8 * (lane & 7);                               \
      if (KVNT) vraw[x] = __builtin_bit_cast(uint4, __builtin_nontemporal_load((const u32x4_kv*)vp_)); \
      else vraw[x] = *(const uint4*)vp_;                                                        \
    }                                                                                           \
  }
  // queries: row lr (clamped), head dimensions 32s + 8*lq .. +8, scaled, as bf16 hi + lo
  bf16x8 qhi[2], qlo[2];
  if constexpr (QU > 0) {
    constexpr int K = 128 * QU, KSTEPS = K / 32, NV4 = 64 * QU, J = QU > 4 ? 2 : 1;
    // LDS that the key loop and the final merge use later: statistics and gain / bias in vs, the waves' partial sums in o_s
    float* st_s = (float*)&vs[0][0][0];          // [K/16][16][2]   (<= 8 KB)
    float* gb_s = st_s + 2048;                   // gain at 0, bias at 1024   (8 KB)
    f32x4* red = &o_s[0][0][0];                  // [wave][column tile][lane]
    static_assert(AttnLds::VS_BYTES >= 4 * 4096, "prologue operands fit the V staging area");
    // every global load of the kernel is issued before the first wait: small operands, x, weights, then K / V
    // (named registers: indexed arrays of these were placed in LDS by the compiler)
    const int i0 = tid < NV4 ? tid : 0, i1 = tid + 256 < NV4 ? tid + 256 : 0;
    const float4 gb0 = ((const float4*)(i0 < NV4 / 2 ? qp.g : qp.b))[i0 < NV4 / 2 ? i0 : i0 - NV4 / 2];
    float4 gb1 = gb0;
    if constexpr (J > 1) gb1 = ((const float4*)(i1 < NV4 / 2 ? qp.g : qp.b))[i1 < NV4 / 2 ? i1 : i1 - NV4 / 2];
    // statistics of this sequence's rows: element e = 16 * tile + local row
    // (srows == 16: one partial per 16-column tile, 8 QU of them; otherwise per 64-column block, 2 QU)
    constexpr int JS = QU >= 2 ? QU / 2 : 1;
    const int nparts = qp.srows == 16 ? 8 * QU : 2 * QU, NS2 = 16 * nparts;
    const int row_first = b * p.R + r0;
#define BPD_ST_SRC(e) ((const float2*)qp.stats)[(e) < NS2 ? ((e) >> 4) * qp.srows + row_first + (((e) & 15) < nrows ? ((e) & 15) : nrows - 1) : 0]
    const float2 s0 = BPD_ST_SRC(tid);
    float2 s1 = s0, s2 = s0, s3 = s0;
    if constexpr (JS > 1) s1 = BPD_ST_SRC(tid + 256);
    if constexpr (JS > 2) { s2 = BPD_ST_SRC(tid + 512); s3 = BPD_ST_SRC(tid + 768); }
#undef BPD_ST_SRC
    const int lrc = lr < nrows ? lr : nrows - 1;
    const int grow = row_first + lrc;
    float4 xv[QU][2];
#pragma unroll
    for (int i = 0; i < QU; ++i) {
      const float* xp = qp.x + (long)grow * K + (wave + 4 * i) * 32 + 8 * lq;
      xv[i][0] = *(const float4*)xp; xv[i][1] = *(const float4*)(xp + 4);
    }
    uint4 wf[QU][4];
#pragma unroll
    for (int i = 0; i < QU; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        wf[i][j] = ((const uint4*)qp.W)[((long)(4 * h + j) * KSTEPS + wave + 4 * i) * 64 + lane];
    BPD_LOAD_KV(first)
    __builtin_amdgcn_sched_barrier(0);
    if (tid < NV4) *(float4*)&gb_s[tid < NV4 / 2 ? 4 * tid : 1024 + 4 * (tid - NV4 / 2)] = gb0;
    if (J > 1 && tid + 256 < NV4) {
      const int idx = tid + 256;
      *(float4*)&gb_s[idx < NV4 / 2 ? 4 * idx : 1024 + 4 * (idx - NV4 / 2)] = gb1;
    }
    if (tid < NS2) ((float2*)st_s)[tid] = s0;
    if constexpr (JS > 1) ((float2*)st_s)[tid + 256] = s1;
    if constexpr (JS > 2) { ((float2*)st_s)[tid + 512] = s2; ((float2*)st_s)[tid + 768] = s3; }
    __syncthreads();
    float sm = 0.f, sq = 0.f;                    // row statistics: this lane adds partials lq, lq + 4, ...
#pragma unroll
    for (int i = 0; i < 2 * QU; ++i) {
      const int part = lq + 4 * i;
      const float2 v = ((const float2*)st_s)[(part < nparts ? part : 0) * 16 + lrc];
      sm += part < nparts ? v.x : 0.f; sq += part < nparts ? v.y : 0.f;
    }
    sm += __shfl_xor(sm, 16, 64); sm += __shfl_xor(sm, 32, 64);
    sq += __shfl_xor(sq, 16, 64); sq += __shfl_xor(sq, 32, 64);
    const float mu = sm / K;
    const float rstd = 1.0f / sqrtf(fmaxf(sq / K - mu * mu, 0.f) + qp.eps);
    f32x4 qa[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) qa[j] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < QU; ++i) {
      const int col = (wave + 4 * i) * 32 + 8 * lq;
      const float4 g0 = *(const float4*)&gb_s[col], g1 = *(const float4*)&gb_s[col + 4];
      const float4 b0 = *(const float4*)&gb_s[1024 + col], b1 = *(const float4*)&gb_s[1024 + col + 4];
      const uint4 yb = make_uint4(pack_bf16_pair((xv[i][0].x - mu) * rstd * g0.x + b0.x, (xv[i][0].y - mu) * rstd * g0.y + b0.y),
                                  pack_bf16_pair((xv[i][0].z - mu) * rstd * g0.z + b0.z, (xv[i][0].w - mu) * rstd * g0.w + b0.w),
                                  pack_bf16_pair((xv[i][1].x - mu) * rstd * g1.x + b1.x, (xv[i][1].y - mu) * rstd * g1.y + b1.y),
                                  pack_bf16_pair((xv[i][1].z - mu) * rstd * g1.z + b1.z, (xv[i][1].w - mu) * rstd * g1.w + b1.w));
#pragma unroll
      for (int j = 0; j < 4; ++j)
        qa[j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, wf[i][j]), __builtin_bit_cast(bf16x8, yb), qa[j], 0, 0, 0);
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) red[(wave * 4 + j) * 64 + lane] = qa[j];
    __syncthreads();
    {                                            // wave w finishes column tile w: a lane holds row lr, columns 16w + 4lq ..
      f32x4 sum = red[wave * 64 + lane];
#pragma unroll
      for (int w = 1; w < 4; ++w) sum += red[(w * 4 + wave) * 64 + lane];
      *(float4*)&q_s[lr * (DH + 4) + 16 * wave + 4 * lq] = make_float4(sum[0], sum[1], sum[2], sum[3]);
    }
    __syncthreads();
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const float4 q0 = *(const float4*)&q_s[lr * (DH + 4) + 32 * s2 + 8 * lq], q1 = *(const float4*)&q_s[lr * (DH + 4) + 32 * s2 + 8 * lq + 4];
      const float v[8] = {q0.x * p.scale, q0.y * p.scale, q0.z * p.scale, q0.w * p.scale,
                          q1.x * p.scale, q1.y * p.scale, q1.z * p.scale, q1.w * p.scale};
      split_bf16x8(v, qhi[s2], qlo[s2]);
    }
  } else {
    BPD_LOAD_KV(first)
    const int row = r0 + (lr < nrows ? lr : nrows - 1);
    const float* qp = p.Q + ((long)b * p.R + row) * p.d + h * DH + 8 * lq;
    float4 qa[2][2];
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) { qa[s2][0] = *(const float4*)(qp + 32 * s2); qa[s2][1] = *(const float4*)(qp + 32 * s2 + 4); }
    int lim0 = p.limit[b];
    __builtin_amdgcn_sched_barrier(0);            // every global load above is in flight before the first wait
#pragma unroll
    for (int s2 = 0; s2 < 2; ++s2) {
      const float v[8] = {qa[s2][0].x * p.scale, qa[s2][0].y * p.scale, qa[s2][0].z * p.scale, qa[s2][0].w * p.scale,
                          qa[s2][1].x * p.scale, qa[s2][1].y * p.scale, qa[s2][1].z * p.scale, qa[s2][1].w * p.scale};
      split_bf16x8(v, qhi[s2], qlo[s2]);
    }
    (void)lim0;
  }
  int lim = p.limit[b];
  lim = lim < 0 ? 0 : lim;
  int nkeys = p.causal ? lim + r0 + nrows : lim;
  nkeys = nkeys < p.cap ? nkeys : p.cap;
  const int nvis = lr < nrows ? (p.causal ? lim + r0 + lr + 1 : lim) : 0;     // keys row lr may see: nlo .. nvis - 1
  const int nlo = LIMF ? attn_first_key(p, lim + r0 + lr) : 0;
  float m_run = -INFINITY, l_run = 0.f;          // of query row lr over this wave's keys (the 4 lanes of a row agree)
  f32x4 acc[4];                                  // out^T tile dt: head dimensions 16*dt + 4*lq + r, row lr
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) acc[dt] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int c0 = first; c0 < nkeys; c0 += hop) {
    const int k0 = c0 + wave * WK;               // first key of this wave in this chunk
    // V rows of the wave -> LDS (rows past the last key as zeros: their probabilities are zero, their bits unknown)
#pragma unroll
    for (int x = 0; x < 8; ++x) {
      const int kl = 8 * x + (lane >> 3);
      const uint4 v = k0 + kl < nkeys ? vraw[x] : make_uint4(0, 0, 0, 0);
      *(uint2*)&vs[wave][kl][8 * (lane & 7)] = make_uint2(v.x, v.y);
      *(uint2*)&vs[wave][kl][8 * (lane & 7) + 4] = make_uint2(v.z, v.w);
    }
    // scores of the wave's 64 keys: sacc[kt][r] = key k0 + 16*kt + 4*lq + r against query row lr
    f32x4 sacc[4];
    float mx = -INFINITY;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt) {
      f32x4 a = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int s2 = 0; s2 < 2; ++s2) {
        const bf16x8 ka = __builtin_bit_cast(bf16x8, kf[kt][s2]);
        a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qhi[s2], a, 0, 0, 0);
        a = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ka, qlo[s2], a, 0, 0, 0);
      }
      const int kb = k0 + kt * 16 + 4 * lq;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        a[r] = (kb + r < nvis && kb + r >= nlo) ? a[r] : -INFINITY;
        mx = fmaxf(mx, a[r]);
      }
      sacc[kt] = a;
    }
    // K fragments and V rows of this chunk have been used: the next chunk's are requested now and arrive during the
    // softmax and the weighted-value products
    if (c0 + hop < nkeys) BPD_LOAD_KV(c0 + hop)
    mx = fmaxf(mx, __shfl_xor(mx, 16, 64));
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);
    const float alpha = (m_new == -INFINITY) ? 1.f : __expf(m_run - m_new);
    float sum = 0.f;
#pragma unroll
    for (int kt = 0; kt < 4; ++kt)
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const float pv = (m_new == -INFINITY) ? 0.f : __expf(sacc[kt][r] - m_new);
        sacc[kt][r] = pv;
        sum += pv;
      }
    sum += __shfl_xor(sum, 16, 64);
    sum += __shfl_xor(sum, 32, 64);
    l_run = l_run * alpha + sum;
    m_run = m_new;
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) { acc[dt][0] *= alpha; acc[dt][1] *= alpha; acc[dt][2] *= alpha; acc[dt][3] *= alpha; }
    // weighted values: two contractions over 32 keys each.  Position 8*lq + e of the contraction is key
    // 32*j + 4*lq + e (e < 4) or 32*j + 16 + 4*lq + e - 4 (e >= 4): what the score tiles 2j and 2j+1 hold in this lane
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const float pvv[8] = {sacc[2 * j][0], sacc[2 * j][1], sacc[2 * j][2], sacc[2 * j][3],
                            sacc[2 * j + 1][0], sacc[2 * j + 1][1], sacc[2 * j + 1][2], sacc[2 * j + 1][3]};
      bf16x8 phi, plo;
      split_bf16x8(pvv, phi, plo);
#pragma unroll
      for (int dt = 0; dt < 4; ++dt) {
        unsigned short vv[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) vv[e] = vs[wave][32 * j + (e < 4 ? 4 * lq + e : 16 + 4 * lq + e - 4)][16 * dt + lr];
        const bf16x8 va = __builtin_bit_cast(bf16x8, make_uint4((unsigned)vv[0] | ((unsigned)vv[1] << 16), (unsigned)vv[2] | ((unsigned)vv[3] << 16),
                                                                 (unsigned)vv[4] | ((unsigned)vv[5] << 16), (unsigned)vv[6] | ((unsigned)vv[7] << 16)));
        acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, phi, acc[dt], 0, 0, 0);
        acc[dt] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(va, plo, acc[dt], 0, 0, 0);
      }
    }
  }
#undef BPD_LOAD_KV
  // the four waves meet: wave w finishes head dimensions 16w .. 16w+15
#pragma unroll
  for (int dt = 0; dt < 4; ++dt) o_s[wave][dt][lane] = acc[dt];
  if (lq == 0) { m_s[wave][lr] = m_run; l_s[wave][lr] = l_run; }
  __syncthreads();
  float M = -INFINITY;
#pragma unroll
  for (int w = 0; w < 4; ++w) M = fmaxf(M, m_s[w][lr]);
  float L = 0.f;
  f32x4 o = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const float mw = m_s[w][lr];
    const float wgt = (mw == -INFINITY) ? 0.f : __expf(mw - M);
    L = fmaf(l_s[w][lr], wgt, L);
    const f32x4 ow = o_s[w][wave][lane];
    o[0] = fmaf(ow[0], wgt, o[0]); o[1] = fmaf(ow[1], wgt, o[1]); o[2] = fmaf(ow[2], wgt, o[2]); o[3] = fmaf(ow[3], wgt, o[3]);
  }
  const int dim = 16 * wave + 4 * lq;
  if (p.nsplit == 1) {
    if (lr < nrows) {
      const float inv = 1.0f / L;
      bf16_t* op = (bf16_t*)p.out + ((long)b * p.R + r0 + lr) * p.d + h * DH + dim;
      *(uint2*)op = make_uint2((unsigned)f2bf(o[0] * inv) | ((unsigned)f2bf(o[1] * inv) << 16),
                               (unsigned)f2bf(o[2] * inv) | ((unsigned)f2bf(o[3] * inv) << 16));
    }
  } else {
    const int tiles = nz / p.nsplit;
    float* part = p.part + ((((long)b * nheads + h) * tiles + tile) * p.nsplit + split) * (RT * (DH + 2));
    *(float4*)(part + lr * DH + dim) = make_float4(o[0], o[1], o[2], o[3]);
    if (tid < RT) { part[RT * DH + tid] = M; part[RT * DH + RT + tid] = L; }
  }
}
template <bool KVNT, bool LIMF, int QU>
__global__ __launch_bounds__(256) void attention_mfma_kernel(AttnP p, QProjP qp) {
  constexpr int RT = 16, DH = 64, WK = 64, VLD = DH + 4;
  __shared__ __attribute__((aligned(16))) bf16_t vs[4][WK][VLD];
  __shared__ f32x4 o_s[4][4][64];
  __shared__ float m_s[4][RT], l_s[4][RT];
  __shared__ __attribute__((aligned(16))) float q_s[QU > 0 ? RT * (DH + 4) : 4];
  AttnLds sm;
  sm.vs = vs; sm.o_s = o_s; sm.m_s = m_s; sm.l_s = l_s; sm.q_s = q_s;
  attention_mfma_body<KVNT, LIMF, QU>(p, qp, sm, blockIdx.x, blockIdx.y, blockIdx.z, gridDim.x, gridDim.z, threadIdx.x);
}

// Merge of the nsplit partial results of attention_kernel: with M the largest of the partial
// maxima, output = sum_s acc_s e^(m_s - M) / sum_s l_s e^(m_s - M).  Grid (heads, B, row tiles).
template <typename ACT, int DH, int NS>
__global__ __launch_bounds__(256) void attention_combine_kernel(AttnP p) {
  constexpr int RT = 16, PS = RT * (DH + 2), Q4 = DH / 4;       // NS >= p.nsplit: partial results read per thread
  const int h = blockIdx.x, b = blockIdx.y, tile = blockIdx.z, r0 = tile * RT;
  const int nrows = min(RT, p.R - r0);
  const float* part = p.part + (((long)b * gridDim.x + h) * gridDim.z + tile) * p.nsplit * PS;
  // one thread per (row, four head dimensions)
  const int i = threadIdx.x / Q4, c4 = threadIdx.x % Q4;
  if (i >= nrows) return;
  float m[NS], l[NS];
  float4 a[NS];
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const int ss = s < p.nsplit ? s : 0;                 // unconditional loads, unused ones masked below
    m[s] = part[ss * PS + RT * DH + i];
    l[s] = part[ss * PS + RT * DH + RT + i];
    a[s] = *(const float4*)(part + ss * PS + i * DH + 4 * c4);
  }
  float mx = -INFINITY;
#pragma unroll
  for (int s = 0; s < NS; ++s) mx = fmaxf(mx, s < p.nsplit ? m[s] : -INFINITY);
  float den = 0.f;
  float4 num = make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
  for (int s = 0; s < NS; ++s) {
    const float w = (s < p.nsplit && m[s] != -INFINITY) ? __expf(m[s] - mx) : 0.f;
    num.x = fmaf(a[s].x, w, num.x); num.y = fmaf(a[s].y, w, num.y); num.z = fmaf(a[s].z, w, num.z); num.w = fmaf(a[s].w, w, num.w);
    den = fmaf(l[s], w, den);
  }
  ACT* o = (ACT*)p.out + ((long)b * p.R + r0 + i) * p.d + h * DH + 4 * c4;
  if constexpr (sizeof(ACT) == 2) {
    *(uint2*)o = make_uint2((unsigned)f2bf(num.x / den) | ((unsigned)f2bf(num.y / den) << 16),
                            (unsigned)f2bf(num.z / den) | ((unsigned)f2bf(num.w / den) << 16));
  } else {
    o[0] = from_f<ACT>(num.x / den); o[1] = from_f<ACT>(num.y / den); o[2] = from_f<ACT>(num.z / den); o[3] = from_f<ACT>(num.w / den);
  }
}

// ---------------------------------------------------------------------------------------
// Decode state (all arrays on the device, one entry per sequence).
struct StateP {
  int* L;            // committed decoder-cache rows = j + 1
  int* j;            // accepted tokens so far
  int* finished;
  int* max_len;
  int* P;            // [B][kmax]
  int* A;            // [B][kmax][kmax]
  int* accepted;     // [B] k-hat of the last step
  int* out_ids;      // [B][max_out]
  long long* stats;  // [0] seq_steps [1] accepted_total [2] finished [3..19] hist[0..16] [20] live steps
  const int* imposed;  // k-hat to impose: imposed[step * imposed_stride + b], or null
  int imposed_stride;  // B for a whole schedule, 0 for a single step's vector
  int kmax, max_out, eos_id;
  int distance_eps, min_block;
  const int* topn_ok;  // [B][kmax]: proposal i+1 is among the n best of p_1 at row i (null: criterion off)
};

__global__ void fill_u64_kernel(unsigned long long* p, long n, unsigned long long v) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}
__global__ void fill_i32_kernel(int* p, long n, int v) {
  const long i = (long)blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = v;
}

// After the first invocation on the empty prefix: P <- heads at position 0, j = 0, L = 1.
__global__ void prime_kernel(StateP s, const unsigned long long* keys, int B) {
  const int b = blockIdx.x, lane = threadIdx.x;
  if (b >= B) return;
  if (lane < s.kmax) {
    const int a = key_index(keys[b * s.kmax + lane]);
    s.P[b * s.kmax + lane] = a;
    s.A[(b * s.kmax + 0) * s.kmax + lane] = a;
  }
  if (lane == 0) { s.L[b] = 1; s.j[b] = 0; s.finished[b] = 0; s.accepted[b] = 0; }
}

// Top-n acceptance (Section 5.1): is proposal P[b][i+1] among the n best-scoring tokens of p_1 at
// block row i?  logits: [B*k][V] fp32, row b*k + i = head 1 at block row i.  The rank of the
// proposal is the number of tokens that beat it in the (value, lower index first) order of the
// arg-max keys.  Grid (k - 1, B), one workgroup per tested row.
__global__ __launch_bounds__(256) void topn_rank_kernel(const float* logits, int V, const int* P, int kmax, int k, int n,
                                                        int* ok) {
  const int i = blockIdx.x, b = blockIdx.y;
  const float* z = logits + ((long)b * k + i) * V;
  int t = P[b * kmax + i + 1];
  t = t < 0 ? 0 : (t >= V ? V - 1 : t);
  const unsigned long long kt = argmax_key(z[t], (unsigned)t);
  int cnt = 0;
  for (int v = threadIdx.x; v < V; v += 256) cnt += argmax_key(z[v], (unsigned)v) > kt;
  __shared__ int part[4];
  for (int off = 32; off > 0; off >>= 1) cnt += __shfl_xor(cnt, off, 64);
  if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = cnt;
  __syncthreads();
  if (threadIdx.x == 0) ok[b * kmax + i] = (part[0] + part[1] + part[2] + part[3]) < n;
}

// Verify substep for sequence b, one wavefront: lane i (1 <= i < k) holds proposal P_{i+1} in myP and
// a1 = arg-max of p_1 at block row i; returns k-hat before the cut at EOS / max_len: the longest
// prefix whose proposals pass the test (exact match, |P - a1| <= eps, or top-n membership), at
// least min_block, or the imposed value.
// (_v: with the values the decision reads from memory already at hand: topn = topn_ok[b][lane - 1], imposed = the
// step's imposed value; both ignored when the criterion / schedule is off)
__device__ __forceinline__ int verified_length_v(const StateP& s, int k, int lane, int myP, int a1, int topn, int imposed) {
  bool ok = true;
  if (lane >= 1 && lane < k) {
    const int diff = myP > a1 ? myP - a1 : a1 - myP;
    ok = diff <= s.distance_eps || (s.topn_ok && topn);
  }
  const unsigned long long lanes_k = (k >= 64) ? ~0ull : ((1ull << k) - 1ull);
  const unsigned long long bad = (~__ballot(ok)) & lanes_k;
  int khat = bad ? __ffsll((long long)bad) - 1 : k;
  if (khat < s.min_block) khat = s.min_block < k ? s.min_block : k;
  if (s.imposed) khat = imposed < 1 ? 1 : (imposed > k ? k : imposed);
  return khat;
}
__device__ __forceinline__ int verified_length(const StateP& s, int b, int k, int lane, int myP, int a1, int step) {
  const int topn = (s.topn_ok && lane >= 1 && lane < k) ? s.topn_ok[b * s.kmax + lane - 1] : 0;
  const int imposed = s.imposed ? s.imposed[(long)step * s.imposed_stride + b] : 0;
  return verified_length_v(s, k, lane, myP, a1, topn, imposed);
}

// Accept substep, the cut: a verified block ends at (and includes) its first EOS and never exceeds
// the room left under max_len (room = max_len - j); `eos` tells whether the block that remains ends in EOS.
__device__ __forceinline__ int cut_length_v(const StateP& s, int lane, int myP, int khat, int room, bool& eos) {
  eos = false;
  if (s.eos_id >= 0) {
    const unsigned long long eb = __ballot(lane < khat && myP == s.eos_id);
    if (eb) { khat = __ffsll((long long)eb); eos = true; }
  }
  if (khat > room) { khat = room; eos = false; }   // the EOS, if any, was beyond the budget
  return khat;
}
__device__ __forceinline__ int cut_length(const StateP& s, int b, int lane, int myP, int khat, bool& eos) {
  return cut_length_v(s, lane, myP, khat, s.max_len[b] - s.j[b], eos);
}

// Two-phase scoring, between the phases: k-hat (verified, then cut as in the accept kernel) from
// p_1 of the k block rows (keys_h1[b*k + i]), then the block row k-hat of sequence b (bf16 LayerNorm output and its fp32 copy) is gathered for the
// heads 2..k.  Grid B, 256 threads (the first wavefront verifies).
__global__ __launch_bounds__(256) void select_row_kernel(StateP s, const unsigned long long* keys_h1, int k, int step,
                                                         const bf16_t* hn, const float* h, int d, int* sel,
                                                         bf16_t* hn2, float* h2) {
  const int b = blockIdx.x, lane = threadIdx.x & 63;
  __shared__ int row_s;
  if (threadIdx.x < 64) {
    const int myP = lane < k ? s.P[b * s.kmax + lane] : -1;
    const int a1 = (lane >= 1 && lane < k) ? key_index(keys_h1[(long)b * k + lane - 1]) : 0;
    bool eos;
    int khat = verified_length(s, b, k, lane, myP, a1, step);
    khat = cut_length(s, b, lane, myP, khat, eos);   // the row the accept kernel will read
    khat = khat < 1 ? 1 : khat;                      // (a sequence that has already ended keeps its state)
    if (lane == 0) { row_s = khat - 1; sel[b] = khat - 1; }
  }
  __syncthreads();
  const long src = ((long)b * k + row_s) * d, dst = (long)b * d;
  for (int c = threadIdx.x; c < d; c += 256) { hn2[dst + c] = hn[src + c]; h2[dst + c] = h[src + c]; }
}

// Two-phase scoring, after the second phase: the arg-max table in the layout the accept kernel reads.
// Column 0 (head 1) of every block row comes from the first phase, columns 1..k-1 of row sel[b]
// from the second; the other entries stay empty (key 0 reads back as token -1).  Grid B, 256 threads.
__global__ __launch_bounds__(256) void assemble_keys_kernel(const unsigned long long* keys_h1, const unsigned long long* keys2,
                                                            const int* sel, int k, unsigned long long* keys) {
  const int b = blockIdx.x, r = sel[b];
  for (int e = threadIdx.x; e < k * k; e += 256) {
    const int ip = e / k, i = e % k;
    unsigned long long v = 0ull;
    if (i == 0) v = keys_h1[(long)b * k + ip];
    else if (ip == r) v = keys2[(long)b * (k - 1) + i - 1];
    keys[(long)b * k * k + e] = v;
  }
}

// Verify / accept / commit for one sequence per wavefront.
//   keys: [B][k][k] packed argmax keys of this invocation (row i', head i).
//   verify (exact, or |P - argmax| <= eps):  lane i (1 <= i < k) tests proposal P[i] against
//   head 1 at row i-1; the accepted length is the position of the first failing lane (a
//   ballot and a count of trailing ones), forced up to min_block, or replaced by the imposed
//   value; then cut at the first EOS (inclusive) and at max_len; append; L += k-hat commits
//   the cache rows of the accepted tokens (rejected rows are simply overwritten next step);
//   P <- row k-hat of the table.
//   step: row of the imposed schedule; live_step: steps made since the last bpd_encode (for the step counter).
__global__ __launch_bounds__(64) void accept_kernel(StateP s, const unsigned long long* keys, int k, int B,
                                                    int commit, int step, int* accepted_out, int live_step) {
  const int b = blockIdx.x, lane = threadIdx.x;
  if (b >= B) return;
  for (int e = lane; e < k * k; e += 64) {
    const int ip = e / k, i = e % k;
    s.A[(b * s.kmax + ip) * s.kmax + i] = key_index(keys[(long)b * k * k + e]);
  }
  if (!commit) return;
  if (s.finished[b]) {
    if (lane == 0) { s.accepted[b] = 0; if (accepted_out) accepted_out[b] = 0; }
    return;
  }
  const int myP = lane < k ? s.P[b * s.kmax + lane] : -1;
  const int a1 = (lane >= 1 && lane < k) ? key_index(keys[(long)b * k * k + (lane - 1) * k + 0]) : 0;
  int khat = verified_length(s, b, k, lane, myP, a1, step);
  bool eos = false;
  const int j = s.j[b];
  khat = cut_length(s, b, lane, myP, khat, eos);
  if (lane < khat) s.out_ids[(long)b * s.max_out + j + lane] = myP;
  const int nextP = lane < k ? key_index(keys[(long)b * k * k + (khat - 1) * k + lane]) : 0;
  if (lane < k) s.P[b * s.kmax + lane] = nextP;
  if (lane == 0) {
    const int fin = eos || (j + khat >= s.max_len[b]);
    s.j[b] = j + khat;
    s.L[b] = s.L[b] + khat;
    s.finished[b] = fin;
    s.accepted[b] = khat;
    if (accepted_out) accepted_out[b] = khat;
    atomicAdd((unsigned long long*)&s.stats[0], 1ull);
    atomicAdd((unsigned long long*)&s.stats[1], (unsigned long long)khat);
    if (fin) atomicAdd((unsigned long long*)&s.stats[2], 1ull);
    atomicAdd((unsigned long long*)&s.stats[3 + khat], 1ull);
    atomicMax((unsigned long long*)&s.stats[20], (unsigned long long)(live_step + 1));   // steps with a live sequence
  }
}

// accept_kernel followed, in the same launch, by the embedding of the next block (embed_stats_kernel; bf16, d <= 1024):
// the step is a chain of dependent kernels and each one saved counts.  One
// workgroup of 16 waves per sequence: wave 0 verifies / accepts / commits, then every wave embeds four 16-column tiles of
// the sequence's k next rows (token i = new proposal i, position = new L + i) with their partial LayerNorm statistics,
// exactly as embed_stats_kernel would at the start of the next step, and the sequence's k*k arg-max keys are cleared
// for the next vocabulary projection.
// stats: srows = 16: [(tile * 16 + row) * 2] per 16-column tile; otherwise srows = B * k rows and one entry per
// 64-column block, [(block * srows + row) * 2]; xb (may be null):
// bf16 copy of the rows as well.
__global__ __launch_bounds__(1024) void accept_embed_kernel(StateP s, unsigned long long* keys, int k, int B, int step,
                                                            int* accepted_out, int d, const bf16_t* E, int V,
                                                            const float* pos, float scale, float* x, float* stats,
                                                            int srows, bf16_t* xb, int live_step) {
  __shared__ int tok_s[16];
  __shared__ int L_s;
  __shared__ int A_s[256];                       // the sequence's k x k arg-max table
  const int b = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if (b >= B) return;
  if (wave == 0) {
    // one round trip for all the state the decision reads (the chain of dependent loads of accept_kernel costs more
    // than its arithmetic); the table then passes through LDS, so row k-hat needs no second trip
    const int kk = k * k;
    unsigned long long kv[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) kv[q] = keys[(long)b * kk + (lane + 64 * q < kk ? lane + 64 * q : 0)];
    const int myP_raw = s.P[b * s.kmax + (lane < k ? lane : 0)];
    const int fin0 = s.finished[b], j = s.j[b], max_len = s.max_len[b], L0 = s.L[b];
    const int imp_raw = s.imposed ? s.imposed[(long)step * s.imposed_stride + b] : 0;
    const int topn_raw = s.topn_ok ? s.topn_ok[b * s.kmax + ((lane >= 1 && lane < k) ? lane - 1 : 0)] : 0;
    __builtin_amdgcn_sched_barrier(0);
    const int myP = lane < k ? myP_raw : -1;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int e = lane + 64 * q;
      if (e < kk) {
        const int a = key_index(kv[q]);
        A_s[e] = a;
        s.A[(b * s.kmax + e / k) * s.kmax + e % k] = a;
      }
    }
    if (fin0) {
      if (lane == 0) { s.accepted[b] = 0; if (accepted_out) accepted_out[b] = 0; L_s = L0; }
      if (lane < k) tok_s[lane] = myP;
    } else {
      // (a wave's LDS accesses execute in order: the table written above is read back without a barrier)
      const int a1 = (lane >= 1 && lane < k) ? A_s[(lane - 1) * k] : 0;
      int khat = verified_length_v(s, k, lane, myP, a1, topn_raw, imp_raw);
      bool eos = false;
      khat = cut_length_v(s, lane, myP, khat, max_len - j, eos);
      if (lane < khat) s.out_ids[(long)b * s.max_out + j + lane] = myP;
      const int nextP = lane < k ? A_s[(khat > 0 ? khat - 1 : 0) * k + lane] : 0;
      if (lane < k) { s.P[b * s.kmax + lane] = nextP; tok_s[lane] = nextP; }
      if (lane == 0) {
        const int fin = eos || (j + khat >= max_len);
        const int Ln = L0 + khat;
        s.j[b] = j + khat;
        s.L[b] = Ln;
        L_s = Ln;
        s.finished[b] = fin;
        s.accepted[b] = khat;
        if (accepted_out) accepted_out[b] = khat;
        atomicAdd((unsigned long long*)&s.stats[0], 1ull);
        atomicAdd((unsigned long long*)&s.stats[1], (unsigned long long)khat);
        if (fin) atomicAdd((unsigned long long*)&s.stats[2], 1ull);
        atomicAdd((unsigned long long*)&s.stats[3 + khat], 1ull);
        atomicMax((unsigned long long*)&s.stats[20], (unsigned long long)(live_step + 1));   // steps with a live sequence
      }
    }
  }
  __syncthreads();
  for (int e = tid; e < k * k; e += 1024) keys[(long)b * k * k + e] = 0ull;
  // rows b*k .. b*k + k - 1 of the next block
  const int i = lane & 15, ic = i < k ? i : k - 1;
  int t = tok_s[ic];
  t = t < 0 ? 0 : (t >= V ? V - 1 : t);
  const int position = L_s + ic;
  const int row = b * k + ic;
  const int ksteps = d >> 5, ntiles = d >> 4;
  // srows == 16: statistics per 16-column tile (tiles wave, wave + 16, ..); otherwise per 64-column block: the wave's
  // four tiles are block `wave` and their sums are added up here
  const bool per_block = srows != 16;
  float bs = 0.f, bq = 0.f;
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int tile = per_block ? 4 * wave + q : wave + 16 * q;
    if (tile >= ntiles) break;                   // the same for the whole wave
    const int c0 = tile * 16 + (lane >> 4) * 4;
    const float4 pv = *(const float4*)(pos + (long)position * d + c0);
    const long tl = (long)(t >> 4) * ksteps + (c0 >> 5);
    const int ln = 16 * ((c0 & 31) >> 3) + (t & 15);
    const uint2 raw = *(const uint2*)(E + (tl * 64 + ln) * 8 + (c0 & 7));
    float v[4] = {pv.x, pv.y, pv.z, pv.w};
    v[0] += scale * __uint_as_float(raw.x << 16); v[1] += scale * __uint_as_float(raw.x & 0xFFFF0000u);
    v[2] += scale * __uint_as_float(raw.y << 16); v[3] += scale * __uint_as_float(raw.y & 0xFFFF0000u);
    float sv = (v[0] + v[1]) + (v[2] + v[3]);
    float qv = (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]);
    sv += __shfl_xor(sv, 16, 64); sv += __shfl_xor(sv, 32, 64);
    qv += __shfl_xor(qv, 16, 64); qv += __shfl_xor(qv, 32, 64);
    bs += sv; bq += qv;
    if (!per_block && lane < 16 && i < k) ((float2*)stats)[(long)tile * srows + row] = make_float2(sv, qv);
    if (i < k) {
      *(float4*)(x + (long)row * d + c0) = make_float4(v[0], v[1], v[2], v[3]);
      if (xb) *(uint2*)(xb + (long)row * d + c0) = make_uint2((unsigned)f2bf(v[0]) | ((unsigned)f2bf(v[1]) << 16), (unsigned)f2bf(v[2]) | ((unsigned)f2bf(v[3]) << 16));
    }
  }
  if (per_block && 4 * wave < ntiles && lane < 16 && i < k) ((float2*)stats)[(long)wave * srows + row] = make_float2(bs, bq);
}

// ---------------------------------------------------------------------------------------
// Machine peaks, measured the way the step's kernels use the machine (bpd_measure_*).
// Streaming read: every thread sums 16-byte words of a buffer, grid-stride, nothing written
// (the impossible comparison keeps the loads alive).
__global__ __launch_bounds__(256) void peak_read_kernel(const uint4* src, long n16, unsigned* sink) {
  unsigned acc = 0;
  constexpr int U = 8;                           // 16-byte loads in flight per lane (4: 6.2 TB/s, 8: 6.3 TB/s)
  const long stride = (long)gridDim.x * 256 * U;
  for (long i = (long)blockIdx.x * 256 * U + threadIdx.x; i < n16; i += stride) {
    uint4 v[U];
#pragma unroll
    for (int j = 0; j < U; ++j) v[j] = src[i + 256 * j < n16 ? i + 256 * j : i];
#pragma unroll
    for (int j = 0; j < U; ++j) acc ^= v[j].x ^ v[j].y ^ v[j].z ^ v[j].w;
  }
  if (acc == 0x9E3779B9u && n16 < 0) sink[0] = acc;
}

// Matrix pipe: 16 independent accumulators per wave, v_mfma_f32_16x16x32_bf16 back to back with
// pseudo-random bf16 operands (the sustained clock depends on the data), nothing else.
__global__ __launch_bounds__(256) void peak_mfma_kernel(float* sink, int iters, unsigned seed) {
  f32x4 acc[16];
#pragma unroll
  for (int i = 0; i < 16; ++i) acc[i] = f32x4{0.f, 0.f, 0.f, 0.f};
  bf16x8 a[4], b[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    unsigned h = (threadIdx.x * 4 + j + blockIdx.x * 1024) * 2654435761u + seed;
    unsigned w[8];
#pragma unroll
    for (int q = 0; q < 8; ++q) { h ^= h >> 15; h *= 2246822519u; h ^= h >> 13; w[q] = (h & 0x807F807Fu) | 0x3D003D00u | ((h >> 3) & 0x01800180u); }
    a[j] = __builtin_bit_cast(bf16x8, make_uint4(w[0], w[1], w[2], w[3]));
    b[j] = __builtin_bit_cast(bf16x8, make_uint4(w[4], w[5], w[6], w[7]));
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 16; ++i) acc[i] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(a[i & 3], b[(i >> 2) & 3], acc[i], 0, 0, 0);
  }
  float sum = 0.f;
#pragma unroll
  for (int i = 0; i < 16; ++i) sum += acc[i][0] + acc[i][1] + acc[i][2] + acc[i][3];
  if (sum == 12345.678f) sink[0] = sum;
}

