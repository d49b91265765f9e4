// Work distribution and barrier schedule of the decoder stack kernel (bpd_stack.h), free of any HIP dependency so
// that the host can check it: the compute waves and the helper waves of a worker run different code and must arrive
// at exactly the same sequence of workgroup barriers, or the workgroup never finishes.  Both roles are written as
// walkers over a visitor: the kernel's visitors do the work, a host test's visitors record the barriers
// (tests/test_host_logic.py compiles this file with the system compiler under the address / undefined sanitizers).
#pragma once

#if defined(__HIPCC__)
#define BPD_HD __host__ __device__
#else
#define BPD_HD
#endif

constexpr int STACK_MAX_LAYERS = 8;
constexpr int STACK_FLAG_STRIDE = 64;      // flag words per operator instance (>= workers)
constexpr int STACK_OPS = 8;               // operators per layer: QKV, self-attention, its output projection, cross query
                                           // projection, cross-attention, its output projection, FFN in, FFN out
constexpr int STACK_BAR_A = 0;             // a GEMM operator's input block is staged in LDS
constexpr int STACK_BAR_B = 1;             // the worker's partial sums of a GEMM operator are in LDS
constexpr int STACK_BAR_ATT = 2;           // the barrier inside one attention item

// exchange buffers of one layer (16 rows each): q, attn, x1, q2, attn2, x2, ffh, x3 (byte offsets)
struct StackEx { long q, attn, x1, q2, attn2, x2, ffh, x3, total; };
BPD_HD inline StackEx stack_ex(int d, int F) {
  StackEx e;
  const long f = 16L * d * 4, h = 16L * d * 2;
  e.q = 0; e.attn = e.q + f; e.x1 = e.attn + h; e.q2 = e.x1 + f; e.attn2 = e.q2 + f; e.x2 = e.attn2 + h;
  e.ffh = e.x2 + f; e.x3 = e.ffh + 16L * F * 2; e.total = e.x3 + f;
  return e;
}
constexpr int STACK_LAYER_TABLE_BYTES = STACK_MAX_LAYERS * 18 * 8;     // 18 pointers per layer (StackLayerP)

struct StackShape {
  int n_layers, d, F, heads, B, M;         // M = block rows (<= 16)
  int workers;                              // workgroups of the working XCD
  int KU;                                   // k-steps of 32 per compute wave and unit (= d / 128)
};
struct StackIt { int layer, g, jl, c; };   // a unit: layer, GEMM operator g, tile of the worker, K chunk

// GEMM operators of a layer in order: g = 0 QKV, 1 self-attention output, 2 cross query, 3 cross-attention output,
// 4 FFN in, 5 FFN out; in the layer's chain of 8 operators they sit at 0, 2, 3, 5, 6, 7 (1 and 4 are the attentions).
BPD_HD inline int stack_gemm_K(const StackShape& s, int g) { return g == 5 ? s.F : s.d; }
BPD_HD inline int stack_gemm_tiles(const StackShape& s, int g) { return (g == 0 ? 3 * s.d : (g == 4 ? s.F : s.d)) / 16; }
BPD_HD inline int stack_gemm_of_op(int op) { return op == 0 ? 0 : (op <= 3 ? op - 1 : op - 2); }      // op not 1, 4
BPD_HD inline int stack_tiles_of(int ntiles, int rank, int workers) {
  return rank < ntiles ? (ntiles - rank + workers - 1) / workers : 0;
}
BPD_HD inline int stack_items_of(const StackShape& s, int rank) {        // attention items (head, sequence) of a worker
  const int items = s.heads * s.B;
  return rank < items ? (items - rank + s.workers - 1) / s.workers : 0;
}
BPD_HD inline int stack_chunks(const StackShape& s, int g) { return (stack_gemm_K(s, g) + 128 * s.KU - 1) / (128 * s.KU); }
// workers that produce the output of operator `op` (the flags a consumer polls)
BPD_HD inline int stack_producers(const StackShape& s, int op) {
  const int units = (op == 1 || op == 4) ? s.heads * s.B : stack_gemm_tiles(s, stack_gemm_of_op(op));
  return units < s.workers ? units : s.workers;
}
// LDS: activations [M][K + 8] bf16 at 0, then the partial sums [tile of the worker][compute wave][lane] f32x4;
// `attn_bytes`: what one attention item needs (from 0); 16 bytes at the end hold the helpers' arrival counter
BPD_HD inline int stack_part_offset(int M, int K) { return (M * (K + 8) * 2 + 15) & ~15; }
BPD_HD inline int stack_lds_need(const StackShape& s, int attn_bytes) {
  int need = attn_bytes;
  for (int g = 0; g < 6; ++g) {
    const int tl = (stack_gemm_tiles(s, g) + s.workers - 1) / s.workers;
    const int b = stack_part_offset(s.M, stack_gemm_K(s, g)) + tl * 4096;
    need = b > need ? b : need;
  }
  return ((need + 15) & ~15) + 16;
}

// moves `it` to the first unit of worker `rank` at or after it (layer == n_layers: none left)
BPD_HD inline void stack_settle(const StackShape& s, int rank, StackIt& it) {
  while (it.layer < s.n_layers) {
    const int ntl = stack_tiles_of(stack_gemm_tiles(s, it.g), rank, s.workers), nch = stack_chunks(s, it.g);
    if (it.jl < ntl && it.c < nch) return;
    if (it.jl < ntl) { it.c = 0; ++it.jl; continue; }
    it.c = 0; it.jl = 0;
    if (++it.g == 6) { it.g = 0; ++it.layer; }
  }
}
BPD_HD inline void stack_advance(const StackShape& s, int rank, StackIt& it) { ++it.c; stack_settle(s, rank, it); }

// Compute waves.  The visitor provides
//   void barrier(int kind);
//   template <int S> void load(const StackIt& unit);                 request the unit's weights into register slot S
//   template <int S> void consume(const StackIt& unit, bool last);   multiply slot S; last: the tile's final chunk
// Four units are in flight; past the last unit the last one is requested again (the loads stay unconditional).
template <class V>
BPD_HD inline void stack_compute_walk(const StackShape& s, int rank, V& v) {
  const int natt = stack_items_of(s, rank);
  StackIt pf{0, 0, 0, 0};
  stack_settle(s, rank, pf);
  if (pf.layer >= s.n_layers) {                   // no tile at all: only the attention items' barriers, if any
    for (int l = 0; l < s.n_layers; ++l)
      for (int i = 0; i < 2 * natt; ++i) v.barrier(STACK_BAR_ATT);
    return;
  }
  StackIt last_valid = pf;
#define BPD_STACK_LOAD(S)                                            \
  {                                                                  \
    if (pf.layer < s.n_layers) last_valid = pf;                      \
    v.template load<S>(last_valid);                                  \
    if (pf.layer < s.n_layers) stack_advance(s, rank, pf);           \
  }
  BPD_STACK_LOAD(0) BPD_STACK_LOAD(1) BPD_STACK_LOAD(2) BPD_STACK_LOAD(3)
  StackIt cs{0, 0, 0, 0};
  stack_settle(s, rank, cs);
  // the attention operators sit before g = 1 and g = 3: their barriers between two chain positions (layer * 6 + g)
  auto attention_barriers = [&](int from, int to) {
    for (int q = from + 1; q <= to; ++q) {
      const int g = q % 6;
      if (g == 1 || g == 3)
        for (int i = 0; i < natt; ++i) v.barrier(STACK_BAR_ATT);
    }
  };
  attention_barriers(-1, cs.layer * 6 + cs.g);
#define BPD_STACK_STEP(S)                                                                              \
  {                                                                                                    \
    if (cs.layer < s.n_layers) {                                                                       \
      const int ntl = stack_tiles_of(stack_gemm_tiles(s, cs.g), rank, s.workers);                      \
      const bool last = cs.c == stack_chunks(s, cs.g) - 1;                                             \
      if (cs.jl == 0 && cs.c == 0) v.barrier(STACK_BAR_A);                                             \
      v.template consume<S>(cs, last);                                                                 \
      if (last && cs.jl == ntl - 1) v.barrier(STACK_BAR_B);                                            \
      const int from = cs.layer * 6 + cs.g;                                                            \
      stack_advance(s, rank, cs);                                                                      \
      const int to = cs.layer < s.n_layers ? cs.layer * 6 + cs.g : s.n_layers * 6 - 1;                 \
      if (to != from) attention_barriers(from, to);                                                    \
    }                                                                                                  \
    BPD_STACK_LOAD(S)                                                                                  \
  }
  while (cs.layer < s.n_layers) { BPD_STACK_STEP(0) BPD_STACK_STEP(1) BPD_STACK_STEP(2) BPD_STACK_STEP(3) }
#undef BPD_STACK_STEP
#undef BPD_STACK_LOAD
}

// Helper waves.  The visitor provides
//   void attention(int layer, int op, int inst, int producers);   all items of the worker: wait for the producers of the
//        previous operator, then per item ONE workgroup barrier (STACK_BAR_ATT), then raise the worker's flag
//   void gemm(int layer, int op, int inst, int producers, int tiles);   request what does not depend on the input, wait
//        for the producers (inst > 0), stage the input block, barrier A, barrier B, finish the tiles, raise the flag
// (what an operator keeps in registers between its phases stays local to one call)
template <class V>
BPD_HD inline void stack_helper_walk(const StackShape& s, int rank, V& v) {
  const int natt = stack_items_of(s, rank);
  for (int layer = 0; layer < s.n_layers; ++layer)
    for (int op = 0; op < STACK_OPS; ++op) {
      const int inst = layer * STACK_OPS + op;
      const int prev_prod = inst > 0 ? stack_producers(s, (op + STACK_OPS - 1) % STACK_OPS) : 0;
      if (op == 1 || op == 4) {
        if (natt > 0) v.attention(layer, op, inst, prev_prod);
        continue;
      }
      const int ntl = stack_tiles_of(stack_gemm_tiles(s, stack_gemm_of_op(op)), rank, s.workers);
      if (ntl > 0) v.gemm(layer, op, inst, prev_prod, ntl);
    }
}
