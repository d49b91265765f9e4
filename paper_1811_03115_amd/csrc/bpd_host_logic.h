// Host-side logic of libbpd that decides sizes and launch shapes: workspace layout, tile choice of the LDS-staged
// GEMM, split factors.  No HIP dependency: bpd.hip includes it, and tests/host/host_logic_check.cpp compiles it with the
// system compiler under the address / undefined-behaviour sanitizers (both defects the first GPU runs of this library
// found were in code of this kind: a staging area one tensor did not fit, a dispatch rule that took the wrong kernel).
#pragma once

#include <cstddef>
#include <cstdint>
#include <vector>

#include "../../include/bpd.h"
#include "bpd_stack_sched.h"

namespace {

constexpr size_t ALIGN = 256;

// Scratch of bpd_step_static: the device memory of a step that is neither input nor output nor decode state (arg-max
// keys that the vocabulary projection merges with atomic max, split-KV attention partials, split-K slices), for callers
// that may not allocate and hand over no workspace for it.  One copy per GPU, held until the process ends; every call
// on a GPU shares it, so calls that overlap on one GPU race.  In host code `scratch` is only a handle: the address on
// the current device comes from hipGetSymbolAddress (bpd_create keeps it per device).
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)8 << 20;
constexpr int MAX_DEVICES = 64;
constexpr int KSPLIT_MAX = 16;          // K slices of a split-K GEMM
constexpr int ATTN_LIMF_MIN_WGS = 256;  // attention launches of at least this many workgroups clamp their K/V loads to the length
constexpr int ATTN_PART_SLOTS = 512;   // workgroups of one split attention launch (partial-result slots); 1024 (one 256-key chunk per
                                       // workgroup up to 16 chunks) measured slower: C4 step at 3000 cached rows 0.383 vs 0.362 ms


struct Arena {
  char* base;
  size_t off = 0;
  std::vector<std::pair<size_t, size_t>>* log = nullptr;     // (offset, bytes) of every region, for the host check
  explicit Arena(char* b) : base(b) {}
  void* take(size_t bytes) {
    off = (off + ALIGN - 1) / ALIGN * ALIGN;
    void* p = base + off;
    if (log) log->push_back({off, bytes});
    off += bytes;
    return p;
  }
};

struct LnW { float *g, *b; };
struct EncL { LnW ln1, ln2; void *wqkv, *wo, *w1, *w2; float *b1, *b2; };
// (FoldW: a matrix with the LayerNorm in front of it folded in, see fold_layernorm_kernel; W == nullptr: not kept)
struct FoldW { void* W = nullptr; float* c = nullptr; float* d = nullptr; };
struct DecL { LnW ln1, ln2, ln3; void *wqkv, *wo, *cq, *co, *ckv, *w1, *w2; float *b1, *b2; FoldW f_qkv, f_cq, f_w1; };

struct Layout {
  // weights
  void* emb; float *pos_src, *pos_tgt;
  std::vector<EncL> enc; LnW enc_lnf;
  std::vector<DecL> dec; LnW dec_lnf;
  void *hw1, *hw2; float *hb1, *hb2;
  // caches
  void *selfK, *selfV, *crossK, *crossV;        // [n_dec][B][slots|max_src][d]
  // decoder activations (M = max_batch * k_max rows)
  float *x, *q, *h, *stats_ln, *stats_big, *zeros, *attn_part, *kpart; size_t n_zeros, n_kpart; void *xn, *attn, *ffh, *hn, *H, *O;
  unsigned long long* keys; unsigned long long* keys_h1; float* logits_h1; int* topn_ok;
  void* hn2; float* h2; int* sel;
  // decoder stack kernel (blocks of at most 16 rows): exchange buffers, flags, error word, probe output
  unsigned char* stack_ex = nullptr; unsigned* stack_flags = nullptr; unsigned* stack_err = nullptr; unsigned* xcc_map = nullptr;
  unsigned long long* stack_trace = nullptr; void* stack_layers = nullptr;
  // encoder activations (max_batch * max_src rows)
  float *xe, *qe; void *xen, *ke, *ve, *attne, *ffhe, *mem;
  // state
  int *L, *j, *finished, *max_len, *src_len, *src_ids, *P, *A, *accepted, *out_ids, *step_counter, *imposed1, *sched;
  long long* stats;
  void* staging; size_t staging_bytes;
  size_t total;
};

size_t act_size(const bpd_config& c) { return c.dtype == BPD_BF16 ? 2 : 4; }

bool config_ok(const bpd_config& c) {
  if (c.n_enc_layers < 1 || c.n_dec_layers < 1 || c.d_model < 32 || c.n_heads < 1) return false;
  if (c.d_model % c.n_heads) return false;
  const int dh = c.d_model / c.n_heads;
  if (dh != 16 && dh != 64) return false;
  if (c.dtype == BPD_F32 && dh != 16) return false;     // fp32 mode is for small models only
  if (c.d_model % 32 || c.d_ff % 32 || c.vocab % 16 || c.vocab < 16) return false;
  if (c.d_model > 2048) return false;                   // LayerNorm kernel keeps a row in registers
  if (c.k_max < 1 || c.k_max > 16) return false;
  if (c.max_batch < 1 || c.max_src_len < 1 || c.max_out_len < 1) return false;
  if (c.dtype != BPD_F32 && c.dtype != BPD_BF16) return false;
  if (c.eos_id >= c.vocab || c.ln_eps <= 0.f) return false;
  return true;
}

// Decoder blocks of more than 128 rows run their LayerNorm-then-GEMM pairs as one GEMM on weights with the LayerNorm
// folded in (ROWAFF in bpd_gemm.h); contexts that can see such blocks keep a folded copy of those matrices.
bool fold_kept(const bpd_config& c) {
  return c.dtype == BPD_BF16 && (long)c.max_batch * c.k_max > 128 && c.d_model % 64 == 0 && c.d_model <= 1024;
}

// Shapes the decoder stack kernel is built for (what a step additionally needs is checked per launch)
bool stack_shape_ok(const bpd_config& c) {
  const int d = c.d_model;
  return c.dtype == BPD_BF16 && d == 64 * c.n_heads && (d == 128 || d == 256 || d == 512 || d == 768 || d == 1024) &&
         c.d_ff % 128 == 0 && c.n_dec_layers <= STACK_MAX_LAYERS;
}
constexpr int XCC_MAP_MAX = 1024;          // compute units the placement probe can record

size_t build_layout(const bpd_config& c, char* base, Layout& L, std::vector<std::pair<size_t, size_t>>* log = nullptr) {
  Arena a(base);
  a.log = log;
  const size_t d = c.d_model, F = c.d_ff, V = c.vocab, k = c.k_max, ws = act_size(c), as = act_size(c);
  const size_t slots = (size_t)c.max_out_len + c.k_max + 1;
  auto vec = [&](size_t n) { return (float*)a.take(n * 4); };
  auto mat = [&](size_t kk, size_t nn) { return a.take(kk * nn * ws); };
  auto ln = [&]() { LnW w; w.g = vec(d); w.b = vec(d); return w; };
  L.emb = mat(V, d);
  L.pos_src = vec((size_t)c.max_src_len * d);
  L.pos_tgt = vec(slots * d);
  L.enc.resize(c.n_enc_layers);
  for (auto& e : L.enc) {
    e.ln1 = ln(); e.wqkv = mat(d, 3 * d); e.wo = mat(d, d); e.ln2 = ln();
    e.w1 = mat(d, F); e.b1 = vec(F); e.w2 = mat(F, d); e.b2 = vec(d);
  }
  L.enc_lnf = ln();
  L.dec.resize(c.n_dec_layers);
  for (auto& e : L.dec) {
    e.ln1 = ln(); e.wqkv = mat(d, 3 * d); e.wo = mat(d, d);
    e.ln2 = ln(); e.cq = mat(d, d); e.co = mat(d, d); e.ckv = mat(d, 2 * d);
    e.ln3 = ln(); e.w1 = mat(d, F); e.b1 = vec(F); e.w2 = mat(F, d); e.b2 = vec(d);
  }
  L.dec_lnf = ln();
  if (fold_kept(c)) {
    auto fold = [&](size_t nn) { FoldW f; f.W = mat(d, nn); f.c = vec(nn); f.d = vec(nn); return f; };
    for (auto& e : L.dec) { e.f_qkv = fold(3 * d); e.f_cq = fold(d); e.f_w1 = fold(F); }
  }
  L.hw1 = mat(d, k * F); L.hb1 = vec(k * F); L.hw2 = mat(k * F, d); L.hb2 = vec(k * d);
  const size_t B = c.max_batch, nd = c.n_dec_layers, S = c.max_src_len;
  L.selfK = a.take(nd * B * slots * d * as); L.selfV = a.take(nd * B * slots * d * as);
  L.crossK = a.take(nd * B * S * d * as);    L.crossV = a.take(nd * B * S * d * as);
  const size_t M = B * k;
  L.x = vec(M * d); L.q = vec(M * d); L.h = vec(M * d); L.stats_ln = vec(64 * 16 * 2);
  L.n_zeros = k * F; if (V > L.n_zeros) L.n_zeros = V; if (3 * d > L.n_zeros) L.n_zeros = 3 * d;
  L.zeros = vec(L.n_zeros);
  L.attn_part = vec((size_t)ATTN_PART_SLOTS * 16 * (d / c.n_heads + 2));
  L.n_kpart = (size_t)KSPLIT_MAX * M * d;      // K slices of one residual update of the decoder block
  L.kpart = vec(L.n_kpart);
  L.xn = a.take(M * d * as); L.attn = a.take(M * d * as); L.ffh = a.take(M * F * as);
  L.hn = a.take(M * d * as); L.H = a.take(M * k * F * as); L.O = a.take(M * k * d * as);
  L.keys = (unsigned long long*)a.take(M * k * 8);
  L.keys_h1 = (unsigned long long*)a.take(2 * M * 8);     // keys of head 1 at the step's B*k rows, then the second phase's B*(k-1)
  L.hn2 = a.take(B * d * as); L.h2 = vec(B * d);
  L.logits_h1 = vec(M * V);
  const size_t Me = B * S;
  L.stats_big = vec((size_t)(d / 64 + 1) * (M > Me ? M : Me) * 2);   // per 64-column block and row: sum, sum of squares
  L.xe = vec(Me * d); L.qe = vec(Me * d);
  L.xen = a.take(Me * d * as); L.ke = a.take(Me * d * as); L.ve = a.take(Me * d * as);
  L.attne = a.take(Me * d * as); L.ffhe = a.take(Me * F * as); L.mem = a.take(Me * d * as);
  auto ints = [&](size_t n) { return (int*)a.take(n * 4); };
  L.L = ints(B); L.j = ints(B); L.finished = ints(B); L.max_len = ints(B); L.src_len = ints(B);
  L.src_ids = ints(Me); L.P = ints(B * k); L.A = ints(B * k * k); L.accepted = ints(B); L.topn_ok = ints(B * k); L.sel = ints(B);
  L.out_ids = ints(B * (size_t)c.max_out_len); L.step_counter = ints(1); L.imposed1 = ints(B);
  L.sched = ints(B * (size_t)c.max_out_len);
  L.stats = (long long*)a.take(32 * 8);
  L.xcc_map = (unsigned*)a.take(XCC_MAP_MAX * 4);
  L.stack_err = (unsigned*)a.take(256);
  if (stack_shape_ok(c)) {
    L.stack_ex = (unsigned char*)a.take((size_t)c.n_dec_layers * stack_ex(c.d_model, c.d_ff).total);
    L.stack_flags = (unsigned*)a.take((size_t)c.n_dec_layers * STACK_OPS * STACK_FLAG_STRIDE * 4);
    L.stack_trace = (unsigned long long*)a.take((size_t)STACK_FLAG_STRIDE * c.n_dec_layers * STACK_OPS * 8 * 8);
    L.stack_layers = a.take(STACK_LAYER_TABLE_BYTES);
  }
  size_t biggest = V * d;                    // largest tensor a bpd_load_weights call may stage (elements)
  if (k * d * F > biggest) biggest = k * d * F;
  if (slots * d > biggest) biggest = slots * d;
  if (S * d > biggest) biggest = S * d;
  if (3 * d * d > biggest) biggest = 3 * d * d;
  L.staging_bytes = biggest * 4;
  L.staging = a.take(L.staging_bytes);
  L.total = (a.off + ALIGN - 1) / ALIGN * ALIGN;
  return L.total;
}

constexpr int LDSX_LN_MT_MAX = 3;      // LayerNorm-fused consumers and statistics-writing producers: tiles of at most 48 rows
constexpr int LDSX_LN_M_MAX = 128;     // and blocks of at most 128 rows
constexpr long LDSX_MIN_WGS = 440;
constexpr long LDSX_MIN_WGS_LONGK = 400;   // K >= 2048, fewer than 1024 rows: a workgroup lives long enough that about 1.5 per CU suffice
                                           // (the encoder's 4096-row FFN output: 64-row tiles, 512 workgroups, beat 80-row tiles, 416: encode -2%)
void pick_tile(int M, int N, int K, long zdim, int& mt, int& nt, int mt_max = 8) {
  const int mts[7] = {8, 7, 5, 4, 3, 2, 1};
  long best_area = 0, best_pad = 0;
  mt = 1; nt = (K % 256 == 0) ? 1 : 4;
  for (int n : {1, 2, 4}) {
    if (K % (256 / n) != 0) continue;
    const long cols = (N / 16 + 4 * n - 1) / (4 * n);
    for (int m : mts) {
      if ((n == 1 && m > 3) || m > mt_max) continue;
      if (n == 4 && m >= 4 && K % 128 != 0) continue;       // these tiles walk K two chunks of 64 at a time
      const long bm = 16 * m, mblocks = (M + bm - 1) / bm, pad = mblocks * bm;
      if (mblocks * cols * zdim < (K >= 2048 && M < 1024 ? LDSX_MIN_WGS_LONGK : LDSX_MIN_WGS)) continue;
      const long area = (long)m * n;                  // compared as area * M / pad: padded rows are wasted work
      if (best_area == 0 || area * best_pad > best_area * pad || (area * best_pad == best_area * pad && pad < best_pad)) {
        best_area = area; best_pad = pad; mt = m; nt = n;
      }
    }
  }
}


// In-place residual update with a long K and few output tiles on the LDS-staged kernel: the number of K slices it is
// split into (1: not split): the fewest with which a tile of at least 48 rows still fills the chip; if no slicing gets
// there, the most slices allowed (each at least 512 deep: two chunks; 80 x 2048 x 512 took 4 us more per step as eight
// slices of 256 than as four of 512).  n_kpart: capacity of the slice buffer in floats.
inline int residual_k_slices_of(int d_model, size_t n_kpart, int M, int N, int K) {
  if (N != d_model || K < 2048 || K % 64 != 0) return 1;
  int mt, nt, ns = 1;
  pick_tile(M, N, K, 1, mt, nt);
  if (nt == 1 && mt < 3) {
    for (int t = 2; t <= KSPLIT_MAX && K % (t * 512) == 0 && (size_t)t * M * N <= n_kpart; t *= 2) {
      ns = t;
      pick_tile(M, N, K / t, t, mt, nt);
      if (nt > 1 || mt >= 3) break;
    }
  }
  return ns;
}

// Workgroups per (head, sequence, row tile) of an attention launch: few such pairs over a long cache deal the 256-key
// chunks to several workgroups whose partial softmax results a second kernel merges.
// (the committed length is on the device, but it grows by at most k_max per step: the host knows a bound on the keys)
inline int attention_nsplit_of(const bpd_config& c, long steps, int local_q, int local_m, int cap, int B, int R, int causal) {
  long keys_max = cap;
  if (causal && steps * c.k_max + R < keys_max) keys_max = steps * c.k_max + R;
  // (local attention: the chunks start at the first row's window and end at the last row)
  if (causal && local_q > 0 && (long)local_q + local_m + R < keys_max) keys_max = (long)local_q + local_m + R;
  const int tiles = (R + 15) / 16, chunks = (int)((keys_max + 255) / 256), wgs = c.n_heads * B * tiles;
  int nsplit = 1;
  if (chunks >= 3 && wgs * 2 <= ATTN_PART_SLOTS) {
    nsplit = ATTN_PART_SLOTS / wgs;
    if (nsplit > chunks) nsplit = chunks;
    if (nsplit > 16) nsplit = 16;
  }
  return nsplit;
}

}  // namespace
