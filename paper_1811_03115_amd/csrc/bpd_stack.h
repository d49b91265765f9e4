// The decoder layers of one step as ONE kernel running on ONE XCD (blocks of at most 16 rows, bf16, 64-wide heads).
//
// Why: with a block of <= 16 rows the decoder stack is a chain of ~42 dependent small operators (per layer: QKV
// projection, self-attention, output projection, cross-attention query projection, cross-attention, output projection,
// two FFN layers; Section 6 of the paper adds nothing to the layers themselves).  As separate kernels each link costs
// 5-7 us (launch, cache write-back / invalidate at the kernel boundary, first memory round trip), and handing the
// 40 KB block between workgroups of DIFFERENT XCDs inside one kernel costs as much (their L2s are not coherent: the
// data has to go through memory).  The workgroups of ONE XCD share an L2, and there a hand-over (stores, wait for their
// acknowledgement, an atomic flag per producer; consumers poll the flags with atomics, then load) measures ~1.3 us.
// One XCD streams ~1.2 TB/s, which is what this kernel is bound by; the weights of the operators ahead are requested
// while the current operator waits for its input, so the stream does not stop at the hand-overs.
//
// Structure: grid = one workgroup per CU of the chip; the workgroups that are not on the working XCD exit at once.
// A worker = 4 compute waves + 4 helper waves.
//   compute waves: walk the worker's weight tiles of all operators in order (tile t of an operator belongs to worker
//     t % workers); K is split over the 4 waves; a unit = KU k-steps of 32 per wave; the weights of the next 4 units
//     are always in flight (registers); the activations are MFMA "B" operands read from LDS; per tile the 4 partial
//     sums go to LDS.
//   helper waves: per operator: poll the producers' flags, fetch the input block, apply LayerNorm where the operator
//     has one (two passes over the row in registers), stage it in LDS as bf16, and after the compute waves are done
//     add the partial sums, apply bias / ReLU / residual, store, and raise the worker's flag.  The attention operators
//     run on the helper waves alone (attention_mfma_body), the compute waves only arrive at their barriers.
// Memory rules that make plain loads and stores sufficient inside one XCD: every exchange buffer is written once per
// launch and read only after all its producers' flags are up (so no line is in a vector L1 before it is complete);
// stores are in L2 once their wave's vmcnt is zero; flags are written and polled with L2 atomics.
// Every wait is bounded: after `spin_limit` polls a worker writes the error word and runs on without waiting, and so
// does every worker that sees the word set; the host reports it at its next synchronisation.
#pragma once

#include "bpd_stack_sched.h"

struct StackLayerP {
  const void *wqkv, *wo, *cq, *co, *w1, *w2;             // packed bf16 tiles [n/16][k/32][64][8]
  const float *ln1g, *ln1b, *ln2g, *ln2b, *ln3g, *ln3b;
  const float *b1, *b2;
  void *selfK, *selfV;                                    // [B][slots][d] bf16
  const void *crossK, *crossV;                            // [B][max_src][d] bf16
};
struct StackP {
  const StackLayerP* L;                                   // [n_layers], in device memory (a table in the kernel arguments
                                                          // indexed by the layer would be copied to scratch memory)
  int n_layers, d, F, heads, B, R, M;                     // M = B * R <= 16 block rows
  int slots, max_src;
  const int* Lbase;                                       // [B] committed cache rows of each sequence
  const int* src_len;                                     // [B]
  const float* x_in;                                      // [M][d] embedded block
  float* x_out;                                           // [M][d] output of the last layer
  float* stats_out;                                       // its partial LayerNorm statistics [(tile * 16 + row) * 2]
  unsigned char* ex;                                      // exchange buffers, stack_ex_layer_bytes(d, F) per layer
  unsigned* flags;                                        // [n_layers * STACK_OPS][STACK_FLAG_STRIDE]
  unsigned* err;
  unsigned epoch;                                         // value the flags take in this launch (never 0)
  int spin_limit;
  int xcc, nx, workers;                                   // working XCD, number of XCDs, workgroups on one XCD
  float eps, scale;
  int lds_bytes;                                          // dynamic LDS of the launch (the helpers' counter sits at the end)
  unsigned long long* trace;                              // debugging aid, may be null: [worker][op instance][8] timestamps
};

static_assert(sizeof(StackLayerP) * STACK_MAX_LAYERS == STACK_LAYER_TABLE_BYTES, "layer table size");

__device__ __forceinline__ unsigned stack_xcc_id() {
  unsigned v;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
  return v & 0xF;
}
__global__ void xcc_map_kernel(unsigned* out) {
  if (threadIdx.x == 0) out[blockIdx.x] = stack_xcc_id();
}

__device__ __forceinline__ StackShape stack_shape(const StackP& p, int KU) {
  StackShape s;
  s.n_layers = p.n_layers; s.d = p.d; s.F = p.F; s.heads = p.heads; s.B = p.B; s.M = p.M; s.workers = p.workers; s.KU = KU;
  return s;
}
__device__ __forceinline__ const uint4* stack_gemm_weights(const StackP& p, int layer, int g) {
  const StackLayerP& l = p.L[layer];
  switch (g) {
    case 0: return (const uint4*)l.wqkv;
    case 1: return (const uint4*)l.wo;
    case 2: return (const uint4*)l.cq;
    case 3: return (const uint4*)l.co;
    case 4: return (const uint4*)l.w1;
    default: return (const uint4*)l.w2;
  }
}

// ------------------------------------------------------------------------------------------------ compute waves
// Visitor of stack_compute_walk: the weights of four units in registers (slots 0..3), the activations from LDS.
template <int KU>
struct StackComputeV {
  const StackP& p;
  const StackShape& s;
  unsigned char* smem;
  int rank, lane, cw, lq, rowc;
  uint4 a0[KU], a1[KU], a2[KU], a3[KU];
  f32x4 acc;
  __device__ __forceinline__ StackComputeV(const StackP& p_, const StackShape& s_, unsigned char* smem_, int rank_)
      : p(p_), s(s_), smem(smem_), rank(rank_) {
    lane = threadIdx.x & 63; cw = threadIdx.x >> 6; lq = lane >> 4;
    const int lr = lane & 15;
    rowc = lr < p.M ? lr : p.M - 1;
    acc = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  __device__ __forceinline__ void barrier(int) { __syncthreads(); }
  template <int S> __device__ __forceinline__ uint4 (&slot())[KU] {
    if constexpr (S == 0) return a0;
    else if constexpr (S == 1) return a1;
    else if constexpr (S == 2) return a2;
    else return a3;
  }
  template <int S> __device__ __forceinline__ void load(const StackIt& it) {
    uint4 (&a)[KU] = slot<S>();
    const uint4* W = stack_gemm_weights(p, it.layer, it.g);
    const int ksteps = stack_gemm_K(s, it.g) >> 5;
    const long t = rank + (long)s.workers * it.jl;
#pragma unroll
    for (int i = 0; i < KU; ++i) {
      int ks = 4 * (it.c * KU + i) + cw;
      ks = ks < ksteps ? ks : ksteps - 1;
      a[i] = W[(t * ksteps + ks) * 64 + lane];
    }
  }
  template <int S> __device__ __forceinline__ void consume(const StackIt& it, bool last) {
    uint4 (&a)[KU] = slot<S>();
    const int K = stack_gemm_K(s, it.g), ksteps = K >> 5;
    const bf16_t* xs = (const bf16_t*)smem + (long)rowc * (K + 8) + lq * 8;
#pragma unroll
    for (int i = 0; i < KU; ++i) {
      const int ks = 4 * (it.c * KU + i) + cw;
      if (ks < ksteps) {
        const uint4 b = *(const uint4*)(xs + ks * 32);
        acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a[i]), __builtin_bit_cast(bf16x8, b), acc, 0, 0, 0);
      }
    }
    if (last) {
      f32x4* part = (f32x4*)(smem + stack_part_offset(p.M, K));
      part[(it.jl * 4 + cw) * 64 + lane] = acc;
      acc = f32x4{0.f, 0.f, 0.f, 0.f};
    }
  }
};

// ------------------------------------------------------------------------------------------------ helper waves
// Helper wave 0 polls the producers' flags (one atomic per lane and round); the other helper waves wait for the word it
// then writes in LDS (`go` counts the polls that ended, successfully or not).
__device__ __forceinline__ void stack_poll(const StackP& p, int op_inst, int nprod, int hw, int lane, unsigned* go, unsigned target) {
  if (hw == 0) {
    unsigned* f = p.flags + (long)op_inst * STACK_FLAG_STRIDE;
    int spins = 0;
    while (true) {
      unsigned v = p.epoch;
      if (lane < nprod) v = __hip_atomic_fetch_add(f + lane, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (__all(v == p.epoch)) break;
      if ((++spins & 255) == 0) {
        if (__hip_atomic_load(p.err, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) break;
        if (spins > p.spin_limit) {
          if (lane == 0) atomicCAS(p.err, 0u, 1u + (unsigned)op_inst);
          break;
        }
      }
      __builtin_amdgcn_s_sleep(1);
    }
    if (lane == 0) __hip_atomic_store(go, target, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
  } else {
    int spins = 0;
    while (__hip_atomic_load(go, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP) != target) {
      if (++spins > (p.spin_limit << 2)) break;            // (wave 0 gives up first and writes the word anyway)
      __builtin_amdgcn_s_sleep(1);
    }
  }
}
// All stores of this wave acknowledged; the last of the four helper waves to get here raises the worker's flag.
__device__ __forceinline__ void stack_signal(const StackP& p, int op_inst, int rank, unsigned* cnt, int lane) {
  __builtin_amdgcn_s_waitcnt(0);
  if (lane == 0) {
    const unsigned old = __hip_atomic_fetch_add(cnt, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    if ((old & 3u) == 3u)
      __hip_atomic_exchange(p.flags + (long)op_inst * STACK_FLAG_STRIDE + rank, p.epoch, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// LayerNorm(x) of the block's rows -> bf16 rows in LDS (row stride d + 8).  Wave hw takes rows hw, hw + 4, ...
__device__ __forceinline__ void stack_stage_ln(const StackP& p, const float* x, const float4 (&gv)[4], const float4 (&bv)[4], bf16_t* xs,
                                               int hw, int lane) {
  const int d = p.d, n4 = d >> 2;
#pragma unroll
  for (int half = 0; half < 2; ++half) {                   // rows hw, hw + 4 first, then hw + 8, hw + 12
    if (hw + 8 * half >= p.M) break;                       // the same for the whole wave
    float4 xv[2][4];
#pragma unroll
    for (int rs = 0; rs < 2; ++rs) {
      int r = hw + 8 * half + 4 * rs; r = r < p.M ? r : p.M - 1;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int idx = lane + 64 * i;
        xv[rs][i] = *(const float4*)(x + (long)r * d + 4 * (idx < n4 ? idx : 0));
      }
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int rs = 0; rs < 2; ++rs) {
      const int r = hw + 8 * half + 4 * rs;
      if (r >= p.M) break;                                 // the same for the whole wave
      float s = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float w = (lane + 64 * i) < n4 ? 1.f : 0.f;
        s += w * ((xv[rs][i].x + xv[rs][i].y) + (xv[rs][i].z + xv[rs][i].w));
      }
      s = wave_sum(s);
      const float mu = s / d;
      float q = 0.f;
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float w = (lane + 64 * i) < n4 ? 1.f : 0.f;
        const float e0 = xv[rs][i].x - mu, e1 = xv[rs][i].y - mu, e2 = xv[rs][i].z - mu, e3 = xv[rs][i].w - mu;
        q += w * ((e0 * e0 + e1 * e1) + (e2 * e2 + e3 * e3));
      }
      q = wave_sum(q);
      const float rstd = 1.0f / sqrtf(q / d + p.eps);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int idx = lane + 64 * i;
        if (idx < n4) {
          const float y0 = (xv[rs][i].x - mu) * rstd * gv[i].x + bv[i].x, y1 = (xv[rs][i].y - mu) * rstd * gv[i].y + bv[i].y;
          const float y2 = (xv[rs][i].z - mu) * rstd * gv[i].z + bv[i].z, y3 = (xv[rs][i].w - mu) * rstd * gv[i].w + bv[i].w;
          *(uint2*)(xs + (long)r * (d + 8) + 4 * idx) = make_uint2((unsigned)f2bf(y0) | ((unsigned)f2bf(y1) << 16), (unsigned)f2bf(y2) | ((unsigned)f2bf(y3) << 16));
        }
      }
    }
  }
}
// bf16 rows [M][K] (row stride K in memory) -> LDS rows (row stride K + 8), 16 bytes per thread and load; four rows
// at a time, so that up to eight loads per thread are in flight
__device__ __forceinline__ void stack_stage_copy(const StackP& p, const bf16_t* src, int K, bf16_t* xs, int htid) {
  const int per_row = K >> 3;                              // 16-byte pieces of a row (at most 512)
  for (int r0 = 0; r0 < p.M; r0 += 4) {
    uint4 v00, v01, v10, v11, v20, v21, v30, v31;
    const int c0 = htid, c1 = htid + 256;
    const int cc0 = c0 < per_row ? c0 : 0, cc1 = c1 < per_row ? c1 : 0;
#define BPD_ROW(i) (r0 + (i) < p.M ? r0 + (i) : p.M - 1)
    v00 = ((const uint4*)(src + (long)BPD_ROW(0) * K))[cc0]; v01 = ((const uint4*)(src + (long)BPD_ROW(0) * K))[cc1];
    v10 = ((const uint4*)(src + (long)BPD_ROW(1) * K))[cc0]; v11 = ((const uint4*)(src + (long)BPD_ROW(1) * K))[cc1];
    v20 = ((const uint4*)(src + (long)BPD_ROW(2) * K))[cc0]; v21 = ((const uint4*)(src + (long)BPD_ROW(2) * K))[cc1];
    v30 = ((const uint4*)(src + (long)BPD_ROW(3) * K))[cc0]; v31 = ((const uint4*)(src + (long)BPD_ROW(3) * K))[cc1];
#undef BPD_ROW
    __builtin_amdgcn_sched_barrier(0);
#define BPD_PUT(i, va, vb)                                                                        \
    if (r0 + (i) < p.M) {                                                                         \
      if (c0 < per_row) *(uint4*)(xs + (long)(r0 + (i)) * (K + 8) + 8 * c0) = va;                 \
      if (c1 < per_row) *(uint4*)(xs + (long)(r0 + (i)) * (K + 8) + 8 * c1) = vb;                 \
    }
    BPD_PUT(0, v00, v01) BPD_PUT(1, v10, v11) BPD_PUT(2, v20, v21) BPD_PUT(3, v30, v31)
#undef BPD_PUT
  }
}

// Visitor of stack_helper_walk.
struct StackHelperV {
  const StackP& p;
  unsigned char* smem;
  unsigned* cnt;                           // LDS: [0] arrivals of the helper waves at their signals, [1] polls that ended
  StackEx ex;
  int rank;
  unsigned polls = 0;
  __device__ __forceinline__ StackHelperV(const StackP& p_, unsigned char* smem_, int rank_) : p(p_), smem(smem_), rank(rank_) {
    cnt = (unsigned*)(smem + p.lds_bytes - 16);
    ex = stack_ex(p.d, p.F);
  }
  // (the thread index is made opaque wherever it is used: otherwise every operator's per-lane addresses are computed
  // ahead of the loops and kept in registers, more of them than the register file holds)
  __device__ __forceinline__ static int helper_tid() {
    int t = threadIdx.x - 256;
    asm volatile("" : "+v"(t));
    return t;
  }
  __device__ __forceinline__ unsigned char* layer_ex(int layer) const { return p.ex + (long)layer * ex.total; }
  __device__ __forceinline__ const float* x_before(int layer) const {          // residual stream entering the layer
    return layer == 0 ? p.x_in : (const float*)(layer_ex(layer - 1) + ex.x3);
  }
  __device__ __forceinline__ float* x_after(int layer) const {
    return layer == p.n_layers - 1 ? p.x_out : (float*)(layer_ex(layer) + ex.x3);
  }
  __device__ __forceinline__ void stamp(int inst, int slot) {
    if (p.trace && threadIdx.x == 256) p.trace[((long)rank * (p.n_layers * STACK_OPS) + inst) * 8 + slot] = wall_clock64();
  }
  __device__ __forceinline__ void poll(int inst, int producers) {
    const int t = helper_tid();
    ++polls;
    stack_poll(p, inst, producers, t >> 6, t & 63, cnt + 1, polls);
  }
  __device__ __forceinline__ void signal(int inst) { stack_signal(p, inst, rank, cnt, helper_tid() & 63); }

  __device__ __forceinline__ void attention(int layer, int op, int inst, int producers) {
    const StackLayerP& l = p.L[layer];
    unsigned char* e = layer_ex(layer);
    const bool self = op == 1;
    stamp(inst, 0);
    poll(inst - 1, producers);
    stamp(inst, 1);
    AttnP ap{};
    ap.Q = (const float*)(e + (self ? ex.q : ex.q2)); ap.Kc = self ? l.selfK : l.crossK; ap.Vc = self ? l.selfV : l.crossV;
    ap.out = e + (self ? ex.attn : ex.attn2); ap.cap = self ? p.slots : p.max_src; ap.kv_seq_stride = (long)ap.cap * p.d;
    ap.d = p.d; ap.R = p.R; ap.limit = self ? p.Lbase : p.src_len; ap.causal = self ? 1 : 0; ap.scale = p.scale;
    ap.local_q = 0; ap.local_m = 0; ap.nsplit = 1; ap.part = nullptr;
    const AttnLds sm = AttnLds::carve(smem);
    for (int item = rank; item < p.heads * p.B; item += p.workers)       // one workgroup barrier inside each
      attention_mfma_body<false, false, 0>(ap, QProjP{}, sm, item % p.heads, item / p.heads, 0, p.heads, 1, helper_tid());
    stamp(inst, 5);
    signal(inst);
    stamp(inst, 6);
  }

  __device__ __forceinline__ void gemm(int layer, int op, int inst, int producers, int ntl) {
    const StackLayerP& l = p.L[layer];
    unsigned char* e = layer_ex(layer);
    const int htid = helper_tid(), lane = htid & 63, hw = htid >> 6, lr = lane & 15, lq = lane >> 4;
    const int d = p.d, F = p.F, M = p.M, W = p.workers;
    const int K = op == 7 ? F : d;
    const bool last_layer = layer == p.n_layers - 1;
    bf16_t* xs = (bf16_t*)smem;
    // ---- what does not depend on the operator's input: LayerNorm vectors, bias and residual rows of the tiles this
    // wave finishes (tiles jl = hw, hw + 4: a worker has at most 8).  Requested before the wait.
    float4 pre_g[4], pre_b[4], pre_bias[2], pre_res[2];
    const bool ln = op == 0 || op == 3 || op == 6;
    const float* R = op == 2 ? x_before(layer) : (const float*)(e + (op == 5 ? ex.x1 : ex.x2));
    {
      const int n4 = d >> 2;
      const float* g = op == 0 ? l.ln1g : (op == 3 ? l.ln2g : l.ln3g);
      const float* b = op == 0 ? l.ln1b : (op == 3 ? l.ln2b : l.ln3b);
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int idx = lane + 64 * i;
        if (ln) { pre_g[i] = *(const float4*)(g + 4 * (idx < n4 ? idx : 0)); pre_b[i] = *(const float4*)(b + 4 * (idx < n4 ? idx : 0)); }
      }
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        int jl = hw + 4 * j; jl = jl < ntl ? jl : ntl - 1;
        const int n = (rank + W * jl) * 16 + lq * 4;
        if (op == 6) pre_bias[j] = *(const float4*)(l.b1 + n);
        if (op == 7) pre_bias[j] = *(const float4*)(l.b2 + n);
        if (op == 2 || op == 5 || op == 7) pre_res[j] = *(const float4*)(R + (long)(lr < M ? lr : 0) * d + n);
      }
    }
    stamp(inst, 0);
    if (inst > 0) poll(inst - 1, producers);
    stamp(inst, 1);
    // ---- the input block -> LDS
    if (op == 0) stack_stage_ln(p, x_before(layer), pre_g, pre_b, xs, hw, lane);
    else if (op == 3) stack_stage_ln(p, (const float*)(e + ex.x1), pre_g, pre_b, xs, hw, lane);
    else if (op == 6) stack_stage_ln(p, (const float*)(e + ex.x2), pre_g, pre_b, xs, hw, lane);
    else if (op == 2) stack_stage_copy(p, (const bf16_t*)(e + ex.attn), d, xs, htid);
    else if (op == 5) stack_stage_copy(p, (const bf16_t*)(e + ex.attn2), d, xs, htid);
    else stack_stage_copy(p, (const bf16_t*)(e + ex.ffh), F, xs, htid);
    stamp(inst, 2);
    __syncthreads();                                       // A (STACK_BAR_A)
    stamp(inst, 3);
    __syncthreads();                                       // B (STACK_BAR_B)
    stamp(inst, 4);
    // ---- finish the tiles
    const f32x4* part = (const f32x4*)(smem + stack_part_offset(M, K));
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int jl = hw + 4 * j;
      if (jl >= ntl) break;
      const int t = rank + W * jl, n = t * 16 + lq * 4, m = lr;
      f32x4 s = part[(jl * 4 + 0) * 64 + lane];
#pragma unroll
      for (int w = 1; w < 4; ++w) s += part[(jl * 4 + w) * 64 + lane];
      float v[4] = {s[0], s[1], s[2], s[3]};
      const bool live = m < M;                             // rows past the block hold whatever the clamped operand gave
      if (op == 0) {                                       // queries fp32; keys and values into the cache rows of the block
        if (live) {
          if (n < d) *(float4*)((float*)(e + ex.q) + (long)m * d + n) = make_float4(v[0], v[1], v[2], v[3]);
          else {
            const int b = m / p.R, i = m - b * p.R, col = n < 2 * d ? n - d : n - 2 * d;
            const long row = (long)b * p.slots + p.Lbase[b] + i;
            bf16_t* dst = (bf16_t*)(n < 2 * d ? l.selfK : l.selfV);
            *(uint2*)(dst + row * d + col) = make_uint2((unsigned)f2bf(v[0]) | ((unsigned)f2bf(v[1]) << 16), (unsigned)f2bf(v[2]) | ((unsigned)f2bf(v[3]) << 16));
          }
        }
      } else if (op == 3) {
        if (live) *(float4*)((float*)(e + ex.q2) + (long)m * d + n) = make_float4(v[0], v[1], v[2], v[3]);
      } else if (op == 6) {
        const float4 bs = pre_bias[j];
        if (live)
          *(uint2*)((bf16_t*)(e + ex.ffh) + (long)m * F + n) =
              make_uint2((unsigned)f2bf(fmaxf(v[0] + bs.x, 0.f)) | ((unsigned)f2bf(fmaxf(v[1] + bs.y, 0.f)) << 16),
                         (unsigned)f2bf(fmaxf(v[2] + bs.z, 0.f)) | ((unsigned)f2bf(fmaxf(v[3] + bs.w, 0.f)) << 16));
      } else {                                             // residual updates
        float* Y = op == 2 ? (float*)(e + ex.x1) : (op == 5 ? (float*)(e + ex.x2) : x_after(layer));
        const float4 rv = pre_res[j];
        if (op == 7) {
          const float4 bs = pre_bias[j];
          v[0] += bs.x; v[1] += bs.y; v[2] += bs.z; v[3] += bs.w;
        }
        v[0] += rv.x; v[1] += rv.y; v[2] += rv.z; v[3] += rv.w;
        if (live) *(float4*)(Y + (long)m * d + n) = make_float4(v[0], v[1], v[2], v[3]);
        if (op == 7 && last_layer) {
          // partial LayerNorm statistics of the stored rows per 16-column tile, as the heads' first GEMM reads them
          float sv = live ? (v[0] + v[1]) + (v[2] + v[3]) : 0.f;
          float qv = live ? (v[0] * v[0] + v[1] * v[1]) + (v[2] * v[2] + v[3] * v[3]) : 0.f;
          sv += __shfl_xor(sv, 16, 64); sv += __shfl_xor(sv, 32, 64);
          qv += __shfl_xor(qv, 16, 64); qv += __shfl_xor(qv, 32, 64);
          if (lane < 16) ((float2*)p.stats_out)[t * 16 + lane] = make_float2(sv, qv);
        }
      }
    }
    stamp(inst, 5);
    signal(inst);
    stamp(inst, 6);
  }
};

template <int KU>
__global__ __launch_bounds__(512) void decoder_stack_kernel(StackP p) {
  extern __shared__ __attribute__((aligned(16))) unsigned char stack_smem[];
  if ((int)(blockIdx.x % p.nx) != 0) return;
  if ((int)stack_xcc_id() != p.xcc) {                      // not where the host's probe said: never share data across XCDs
    if (threadIdx.x == 0) atomicCAS(p.err, 0u, 0x80000000u);
    return;
  }
  const int rank = blockIdx.x / p.nx;
  if (rank >= p.workers) return;
  if (threadIdx.x < 4) ((unsigned*)(stack_smem + p.lds_bytes - 16))[threadIdx.x] = 0u;      // arrival counter, poll word
  __syncthreads();
  const StackShape shape = stack_shape(p, KU);
  if (threadIdx.x < 256) {
    StackComputeV<KU> v(p, shape, stack_smem, rank);
    stack_compute_walk(shape, rank, v);
  } else {
    StackHelperV v(p, stack_smem, rank);
    stack_helper_walk(shape, rank, v);
  }
}
