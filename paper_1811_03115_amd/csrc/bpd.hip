// Host side of libbpd: workspace layout, weight loading, and the launch sequences behind
// the C ABI declared in include/bpd.h.  Every step of the method runs in the kernels of
// bpd_kernels.h; this file only orders them on the caller's stream.
#include "../../include/bpd.h"
#include "bpd_kernels.h"
#include "bpd_stack.h"
#include "bpd_host_logic.h"

#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <map>
#include <string>
#include <vector>

namespace {

}  // namespace
static __device__ __align__(256) unsigned char scratch[STATIC_SCRATCH_BYTES];
namespace {
void* g_scratch_ptr[MAX_DEVICES] = {};     // address of `scratch` on each device that has created a context

enum Kind { MAT, MATK_CAT, MATK_SEP, EMB, VEC };
struct WEntry {
  Kind kind;
  int nd; int64_t shape[4];
  void* dst;
  int K, N, ldw, n_off;      // matrices: source K x N, destination row length, column offset
  bool loaded;
};

}  // namespace

struct bpd_ctx {
  bpd_config cfg;
  hipStream_t stream;
  Layout lay;
  std::map<std::string, WEntry> table;
  std::string err;
  int B = 0, S = 0;
  bool encoded = false;
  bool fold_ready = false;        // the folded copies match the loaded weights
  int64_t steps = 0;
  int distance_eps = 0, min_block = 1, top_n = 1, two_phase = 0;
  int local_q = 0, local_m = 0;   // 1D local self-attention in the decoder (0: full causal), bpd_set_local_attention
  int num_cus = 256;                   // compute units of the device the context was created on
  int device = 0;                      // that device's index
  // decoder stack kernel: placement of workgroups on XCDs as probed at creation (workers = 0: not usable), the value
  // its flags take next, and whether a launch has reported a timeout (then the per-operator kernels take over)
  int stack_xcc = 0, stack_nx = 0, stack_workers = 0;
  unsigned stack_epoch = 0;
  bool stack_off = false;
  int x_ready_k = 0;                   // > 0: the last step's accept kernel already embedded the next block of that many rows
  bool weights_exceed_llc = false;     // decoder-side weights read per step > 192 MB (the Infinity Cache holds 256 MB)
  const int* cur_imposed = nullptr; int cur_imposed_stride = 0, cur_imposed_step = 0;   // of the step being run
  int* pinned = nullptr;       // small pinned host scratch
  int prof_phase = 0;
  std::vector<hipEvent_t> prof_ev;
  size_t prof_used = 0;
  int64_t prof_launches = 0;
  // host / device classification of the pointers bpd_step was last given (a virtual address keeps its kind in the
  // unified address space, so the runtime is asked once per distinct pointer, not once per step)
  const void* kind_ptr[4] = {nullptr, nullptr, nullptr, nullptr}; bool kind_host[4] = {false, false, false, false}; int kind_next = 0;
  // a split-K residual update whose slices the next LayerNorm of `pend_x` still has to add
  int pend_slices = 0; const float* pend_bias = nullptr; const float* pend_x = nullptr;
};

namespace {

int fail(bpd_ctx* c, int code, const std::string& msg) {
  if (c) c->err = msg;
  return code;
}
#define HIPCHK(expr)                                                                   \
  do {                                                                                 \
    hipError_t _e = (expr);                                                            \
    if (_e != hipSuccess)                                                              \
      return fail(ctx, BPD_E_HIP, std::string(#expr) + ": " + hipGetErrorString(_e)); \
  } while (0)
#define LAUNCHCHK() HIPCHK(hipGetLastError())

void add_entry(bpd_ctx* ctx, const std::string& name, Kind kind, std::vector<int64_t> shape, void* dst,
               int K = 0, int N = 0, int ldw = 0, int n_off = 0) {
  WEntry e{};
  e.kind = kind; e.nd = (int)shape.size();
  for (int i = 0; i < e.nd; ++i) e.shape[i] = shape[i];
  e.dst = dst; e.K = K; e.N = N; e.ldw = ldw; e.n_off = n_off; e.loaded = false;
  ctx->table[name] = e;
}

void build_table(bpd_ctx* ctx) {
  const bpd_config& c = ctx->cfg;
  Layout& L = ctx->lay;
  const int d = c.d_model, F = c.d_ff, V = c.vocab, k = c.k_max;
  const int slots = c.max_out_len + c.k_max + 1;
  auto ln = [&](const std::string& p, LnW w) {
    add_entry(ctx, p + ".g", VEC, {d}, w.g);
    add_entry(ctx, p + ".b", VEC, {d}, w.b);
  };
  add_entry(ctx, "emb", EMB, {V, d}, L.emb, d, V, V, 0);
  add_entry(ctx, "pos_src", VEC, {c.max_src_len, d}, L.pos_src);
  add_entry(ctx, "pos_tgt", VEC, {slots, d}, L.pos_tgt);
  for (int l = 0; l < c.n_enc_layers; ++l) {
    const std::string p = "enc." + std::to_string(l);
    EncL& e = L.enc[l];
    ln(p + ".ln1", e.ln1); ln(p + ".ln2", e.ln2);
    add_entry(ctx, p + ".self.wq", MAT, {d, d}, e.wqkv, d, d, 3 * d, 0);
    add_entry(ctx, p + ".self.wk", MAT, {d, d}, e.wqkv, d, d, 3 * d, d);
    add_entry(ctx, p + ".self.wv", MAT, {d, d}, e.wqkv, d, d, 3 * d, 2 * d);
    add_entry(ctx, p + ".self.wo", MAT, {d, d}, e.wo, d, d, d, 0);
    add_entry(ctx, p + ".ffn.w1", MAT, {d, F}, e.w1, d, F, F, 0);
    add_entry(ctx, p + ".ffn.b1", VEC, {F}, e.b1);
    add_entry(ctx, p + ".ffn.w2", MAT, {F, d}, e.w2, F, d, d, 0);
    add_entry(ctx, p + ".ffn.b2", VEC, {d}, e.b2);
  }
  ln("enc.lnf", L.enc_lnf);
  for (int l = 0; l < c.n_dec_layers; ++l) {
    const std::string p = "dec." + std::to_string(l);
    DecL& e = L.dec[l];
    ln(p + ".ln1", e.ln1); ln(p + ".ln2", e.ln2); ln(p + ".ln3", e.ln3);
    add_entry(ctx, p + ".self.wq", MAT, {d, d}, e.wqkv, d, d, 3 * d, 0);
    add_entry(ctx, p + ".self.wk", MAT, {d, d}, e.wqkv, d, d, 3 * d, d);
    add_entry(ctx, p + ".self.wv", MAT, {d, d}, e.wqkv, d, d, 3 * d, 2 * d);
    add_entry(ctx, p + ".self.wo", MAT, {d, d}, e.wo, d, d, d, 0);
    add_entry(ctx, p + ".cross.wq", MAT, {d, d}, e.cq, d, d, d, 0);
    add_entry(ctx, p + ".cross.wk", MAT, {d, d}, e.ckv, d, d, 2 * d, 0);
    add_entry(ctx, p + ".cross.wv", MAT, {d, d}, e.ckv, d, d, 2 * d, d);
    add_entry(ctx, p + ".cross.wo", MAT, {d, d}, e.co, d, d, d, 0);
    add_entry(ctx, p + ".ffn.w1", MAT, {d, F}, e.w1, d, F, F, 0);
    add_entry(ctx, p + ".ffn.b1", VEC, {F}, e.b1);
    add_entry(ctx, p + ".ffn.w2", MAT, {F, d}, e.w2, F, d, d, 0);
    add_entry(ctx, p + ".ffn.b2", VEC, {d}, e.b2);
  }
  ln("dec.lnf", L.dec_lnf);
  add_entry(ctx, "head.w1", MATK_CAT, {k, d, F}, L.hw1, d, F, k * F, 0);
  add_entry(ctx, "head.b1", VEC, {k, F}, L.hb1);
  add_entry(ctx, "head.w2", MATK_SEP, {k, F, d}, L.hw2, F, d, d, 0);
  add_entry(ctx, "head.b2", VEC, {k, d}, L.hb2);
}

// ------------------------------------------------------------------------------- launches

template <int MT, int NT, int KS>
void launch_gemm_bf16(const GemmP& p, const Epi& e, int groups, hipStream_t s) {
  const int ntiles = p.N / 16;
  dim3 grid(KS == 4 ? (ntiles + NT - 1) / NT : (ntiles + 4 * NT - 1) / (4 * NT), (p.M + 16 * MT - 1) / (16 * MT), groups);
  hipLaunchKernelGGL((gemm_bf16_kernel<MT, NT, KS>), grid, dim3(256), 0, s, p, e);
}

// ---- skinny path: M <= 16 -------------------------------------------------------------
template <int MT, int NT, bool XLN, bool ARGMAX, int WAVES, int U, int DEPTH, bool STREAM>
void launch_skinny_cfg(const bpd_ctx* ctx, const GemmP& p, const Epi& e_in, const LnP& ln, unsigned long long* keys,
                       float* logits, int groups) {
  hipStream_t s = ctx->stream;
  Epi e = e_in;                                 // the kernel loads bias and residual unconditionally
  if (!e.bias) { e.bias = ctx->lay.zeros; e.bias_g = 0; }
  if (!e.R) { e.R = ctx->lay.zeros; e.ldr = 0; e.r_g = 0; }
  const int ntiles = p.N / 16;
  const int ngroups = (ntiles + NT - 1) / NT;
  // more column-tile groups than CUs: one workgroup per CU walks several of them (a second workgroup on a CU would only
  // start once the first has finished: the kernel fills the register file)
  const int cap = ctx->num_cus;
  const int gx = ngroups > cap ? cap : ngroups;
  dim3 grid(gx, (p.M + 16 * MT - 1) / (16 * MT), groups);
  const size_t lds = (size_t)2 * WAVES * MT * NT * 1024;
  if (ngroups > gx) {
    auto k = skinny_gemm_kernel<MT, NT, XLN, ARGMAX, WAVES, U, DEPTH, STREAM>;
    static bool attr = false;
    if (!attr) { (void)hipFuncSetAttribute((const void*)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); attr = true; }
    hipLaunchKernelGGL(k, grid, dim3(64 * WAVES), lds, s, p, e, ln, keys, logits);
  } else {
    auto k = skinny_gemm_kernel<MT, NT, XLN, ARGMAX, WAVES, U, 0, STREAM>;
    static bool attr = false;
    if (!attr) { (void)hipFuncSetAttribute((const void*)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); attr = true; }
    hipLaunchKernelGGL(k, grid, dim3(64 * WAVES), lds, s, p, e, ln, keys, logits);
  }
}

// One 16-row tile (M <= 16): K split over the waves so that each wave holds all its k-steps.
template <int NT, bool XLN, bool ARGMAX, bool STREAM>
void launch_skinny_s(const bpd_ctx* ctx, const GemmP& p, const Epi& e, const LnP& ln, unsigned long long* keys, float* logits,
                     int groups) {
  // waves x k-steps per wave cover K / 32 without idle slots (an idle slot still costs its clamped load)
  if (XLN && p.K <= 512) launch_skinny_cfg<1, NT, XLN, ARGMAX, 4, 4, 2, STREAM>(ctx, p, e, ln, keys, logits, groups);
  else if (XLN) launch_skinny_cfg<1, NT, XLN, ARGMAX, 8, 4, 2, STREAM>(ctx, p, e, ln, keys, logits, groups);       // K <= 1024
  else if (p.K <= 512) launch_skinny_cfg<1, NT, false, ARGMAX, 4, 4, 2, STREAM>(ctx, p, e, ln, keys, logits, groups);
  else if (p.K <= 1024) launch_skinny_cfg<1, NT, false, ARGMAX, 4, 8, 2, STREAM>(ctx, p, e, ln, keys, logits, groups);
  else if (p.K <= 2048) launch_skinny_cfg<1, NT, false, ARGMAX, 8, 8, 1, STREAM>(ctx, p, e, ln, keys, logits, groups);
  else launch_skinny_cfg<1, NT, false, ARGMAX, 8, 16, 1, STREAM>(ctx, p, e, ln, keys, logits, groups);             // K <= 4096
}
// Streams of at least 32 MB in a model whose per-step weights exceed the last-level cache bypass it.
template <int NT, bool XLN, bool ARGMAX>
void launch_skinny(const bpd_ctx* ctx, const GemmP& p, const Epi& e, const LnP& ln, unsigned long long* keys, float* logits,
                   int groups) {
  const size_t wbytes = (size_t)p.K * p.N * groups * 2;
  if (ctx->weights_exceed_llc && wbytes >= ((size_t)32 << 20)) launch_skinny_s<NT, XLN, ARGMAX, true>(ctx, p, e, ln, keys, logits, groups);
  else launch_skinny_s<NT, XLN, ARGMAX, false>(ctx, p, e, ln, keys, logits, groups);
}

bool skinny_ok(const bpd_ctx* ctx, const GemmP& p) { return ctx->cfg.dtype == BPD_BF16 && p.M <= 16 && p.K <= 4096; }

// ---- streaming path: M <= 16, K = 2048 / 4096, several column tiles per CU ---------------------
// (the heads' output layers at batch 1).  One workgroup per CU walks a contiguous range of at most
// 8 column tiles of one group.
constexpr int STREAM_TILES_MAX = 8;
size_t stream_lds_bytes(const GemmP& p) { return (size_t)16384 + 8192 + 1536 + (size_t)p.M * (p.K + 8) * 2; }
bool stream_ok(const bpd_ctx* ctx, const GemmP& p, const Epi& e, int groups) {
  return skinny_ok(ctx, p) && p.M >= 1 && e.mode == 0 && !e.stats_out && (p.K == 2048 || p.K == 4096) && p.N % 16 == 0 &&
         2L * groups * (p.N / 16) >= 3L * ctx->num_cus && stream_lds_bytes(p) <= (size_t)160 * 1024;
}
template <int U, bool STREAM>
void launch_stream_cfg(const bpd_ctx* ctx, const GemmP& p, const Epi& e_in, int groups) {
  Epi e = e_in;                                 // bias and residual are loaded unconditionally
  if (!e.bias) { e.bias = ctx->lay.zeros; e.bias_g = 0; }
  if (!e.R) { e.R = ctx->lay.zeros; e.ldr = 0; e.r_g = 0; }
  const int ntiles = p.N / 16;
  int gx = ctx->num_cus / groups;
  const int gx_min = (ntiles + STREAM_TILES_MAX - 1) / STREAM_TILES_MAX;
  gx = gx < gx_min ? gx_min : gx;
  gx = gx > ntiles ? ntiles : gx;
  const size_t lds = stream_lds_bytes(p);
  auto k = stream_gemm_kernel<U, STREAM>;
  static size_t attr = 0;                       // per instantiation: allow more than 64 KiB of LDS
  if (attr < lds) { (void)hipFuncSetAttribute((const void*)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); attr = lds; }
  hipLaunchKernelGGL(k, dim3(gx, 1, groups), dim3(512), lds, ctx->stream, p, e);
}
void launch_stream(const bpd_ctx* ctx, const GemmP& p, const Epi& e, int groups) {
  const size_t wbytes = (size_t)p.K * p.N * groups * 2;
  const bool nt = ctx->weights_exceed_llc && wbytes >= ((size_t)32 << 20);
  if (p.K == 4096) { if (nt) launch_stream_cfg<16, true>(ctx, p, e, groups); else launch_stream_cfg<16, false>(ctx, p, e, groups); }
  else { if (nt) launch_stream_cfg<8, true>(ctx, p, e, groups); else launch_stream_cfg<8, false>(ctx, p, e, groups); }
}
// The accept kernel of a step embeds the next step's block (accept_embed_kernel: bf16, at most 64 column tiles)
bool embed_in_accept(const bpd_ctx* ctx) {
  return ctx->cfg.dtype == BPD_BF16 && ctx->cfg.d_model <= 1024;
}
// LayerNorm statistics ride along with the residual stream when the whole block is one MFMA row tile and every GEMM
// that updates the stream is one the skinny kernel takes (it is the one that writes them: K = d_ff must fit it)
bool stats_path(const bpd_ctx* ctx, int M) {
  return ctx->cfg.dtype == BPD_BF16 && M <= 16 && ctx->cfg.d_model <= 1024 && ctx->cfg.d_ff <= 4096;
}

// ---- ldsx path: many rows ---------------------------------------------------------------
template <int MT, int NT, int KC, bool ARGMAX, bool XLN = false, bool STATS = false, bool ROWAFF = false>
void launch_ldsx(const GemmP& p, const Epi& e, unsigned long long* keys, float* logits, int groups, hipStream_t s,
                 const LnP& ln = LnP{}) {
  const int ntiles = p.N / 16;
  dim3 grid((ntiles + 4 * NT - 1) / (4 * NT), (p.M + 16 * MT - 1) / (16 * MT), groups);
  const size_t lds = ldsx_lds_bytes<MT, NT, KC>();
  static bool attr_set = false;                 // per instantiation: allow more than 64 KiB of LDS
  if (!attr_set) {
    (void)hipFuncSetAttribute((const void*)gemm_ldsx_kernel<MT, NT, KC, ARGMAX, XLN, STATS, ROWAFF>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    attr_set = true;
  }
  GemmP q = p;
  q.lx = ldsx_map_of(p.K, KC, p.ksplit, grid.x, grid.y, grid.z);            // (grid.x * grid.y * grid.y * 4 < 2^32 by far: at most a few thousand blocks each way)
  hipLaunchKernelGGL((gemm_ldsx_kernel<MT, NT, KC, ARGMAX, XLN, STATS, ROWAFF>), grid, dim3(256), lds, s, q, e, keys, logits, ln);
}

// Tile of the LDS-staged GEMM: 16*mt rows x 64*nt columns per workgroup, K walked in chunks of
// 256 / 128 / 64 for nt = 1 / 2 / 4 (eight weight fragments per wave in flight either way).
// Chosen: the largest tile that still gives the chip about two workgroups per CU (counting K
// slices and groups); ties go to less row padding, then to the narrower tile (longer chunks).
// With nt = 1 at most 48 rows, so that the two 256-deep staging buffers leave room for three
// workgroups per CU.  If nothing qualifies the smallest tile spreads the work furthest.
// e.stats_out (mode 0, one group, no split over K): the kernel also writes the LayerNorm statistics of its output, which
// only the tiles of at most 48 rows are built for.  Returns whether it did.
// Small tiles fetch bias and residual at kernel entry (Epi::pre_epi): absent operands are replaced by a zero-filled vector.
void prefetch_epilogue(Epi& e, const GemmP& p, int mt, int nt, const float* zeros) {
  if (!zeros || mt * nt > 3 || e.mode != 0 || p.ksplit > 1) return;
  if (!e.bias) { e.bias = zeros; e.bias_g = 0; }
  if (!e.R) { e.R = zeros; e.ldr = 0; e.r_g = 0; }
  e.pre_epi = 1;
}

template <bool ARGMAX>
bool dispatch_ldsx(const GemmP& p, const Epi& e_in, unsigned long long* keys, float* logits, int groups, hipStream_t s,
                   const float* zeros = nullptr) {
  Epi e = e_in;
  int mt, nt;
  const int kslice = p.ksplit > 1 ? p.K / p.ksplit : p.K;
  const bool stats_req = !ARGMAX && e.mode == 0 && e.stats_out != nullptr && groups == 1 && p.ksplit <= 1;
  pick_tile(p.M, p.N, kslice, groups, mt, nt, stats_req ? LDSX_LN_MT_MAX : 8);   // groups = K slices for a split-K launch
  // (the statistics are per 64-column block: every wave of a workgroup must own whole tiles of it)
  const bool stats = stats_req && p.N % (64 * nt) == 0;
  if constexpr (!ARGMAX) prefetch_epilogue(e, p, mt, nt, zeros);
  if constexpr (!ARGMAX) {
    if (stats) {
#define BPD_CASE(MT_, NT_, KC_) if (mt == MT_ && nt == NT_) { launch_ldsx<MT_, NT_, KC_, false, false, true>(p, e, keys, logits, groups, s); return true; }
      BPD_CASE(3, 1, 256) BPD_CASE(2, 1, 256) BPD_CASE(1, 1, 256)
      BPD_CASE(3, 2, 128) BPD_CASE(2, 2, 128) BPD_CASE(1, 2, 128)
      BPD_CASE(3, 4, 64) BPD_CASE(2, 4, 64) BPD_CASE(1, 4, 64)
#undef BPD_CASE
    }
  }
#define BPD_CASE(MT_, NT_, KC_) if (mt == MT_ && nt == NT_) { launch_ldsx<MT_, NT_, KC_, ARGMAX>(p, e, keys, logits, groups, s); return false; }
  BPD_CASE(3, 1, 256) BPD_CASE(2, 1, 256) BPD_CASE(1, 1, 256)
  BPD_CASE(8, 2, 128) BPD_CASE(7, 2, 128) BPD_CASE(5, 2, 128) BPD_CASE(4, 2, 128) BPD_CASE(3, 2, 128) BPD_CASE(2, 2, 128) BPD_CASE(1, 2, 128)
  BPD_CASE(8, 4, 64) BPD_CASE(7, 4, 64) BPD_CASE(5, 4, 64) BPD_CASE(4, 4, 64) BPD_CASE(3, 4, 64) BPD_CASE(2, 4, 64) BPD_CASE(1, 4, 64)
#undef BPD_CASE
  return false;
}

// Y = epilogue(LayerNorm(ln.x) W) on more than 16 rows with the LayerNorm applied while the activations are staged
// (tiles of at most 48 rows: the staging registers).
void dispatch_ldsx_ln(const GemmP& p, const Epi& e_in, const LnP& ln, hipStream_t s, const float* zeros) {
  Epi e = e_in;
  int mt, nt;
  pick_tile(p.M, p.N, p.K, 1, mt, nt, LDSX_LN_MT_MAX);
  prefetch_epilogue(e, p, mt, nt, zeros);
#define BPD_CASE(MT_, NT_, KC_) if (mt == MT_ && nt == NT_) { launch_ldsx<MT_, NT_, KC_, false, true>(p, e, nullptr, nullptr, 1, s, ln); return; }
  BPD_CASE(3, 1, 256) BPD_CASE(2, 1, 256) BPD_CASE(1, 1, 256)
  BPD_CASE(3, 2, 128) BPD_CASE(2, 2, 128) BPD_CASE(1, 2, 128)
  BPD_CASE(3, 4, 64) BPD_CASE(2, 4, 64) BPD_CASE(1, 4, 64)
#undef BPD_CASE
}
// Y = epilogue(LayerNorm(x) W) with the LayerNorm folded into the weights (e.ra_*): X is the raw bf16 copy of x.
void dispatch_ldsx_fold(const GemmP& p, const Epi& e_in, hipStream_t s, const float* zeros) {
  Epi e = e_in;
  int mt, nt;
  pick_tile(p.M, p.N, p.K, 1, mt, nt, LDSX_LN_MT_MAX);
  prefetch_epilogue(e, p, mt, nt, zeros);
#define BPD_CASE(MT_, NT_, KC_) if (mt == MT_ && nt == NT_) { launch_ldsx<MT_, NT_, KC_, false, false, false, true>(p, e, nullptr, nullptr, 1, s); return; }
  BPD_CASE(3, 1, 256) BPD_CASE(2, 1, 256) BPD_CASE(1, 1, 256)
  BPD_CASE(3, 2, 128) BPD_CASE(2, 2, 128) BPD_CASE(1, 2, 128)
  BPD_CASE(3, 4, 64) BPD_CASE(2, 4, 64) BPD_CASE(1, 4, 64)
#undef BPD_CASE
}
bool ldsx_ln_ok(const bpd_ctx* ctx, const GemmP& p) {
  return ctx->cfg.dtype == BPD_BF16 && p.M > 16 && p.K == ctx->cfg.d_model && p.K % 64 == 0 && p.K <= 1024 && p.N % 16 == 0;
}

int residual_k_slices(const bpd_ctx* ctx, const GemmP& p) {
  return residual_k_slices_of(ctx->cfg.d_model, ctx->lay.n_kpart, p.M, p.N, p.K);
}

// Y = epilogue(X W).  bf16 mode: M <= 16 -> skinny kernel; otherwise the LDS-staged kernel
// (K % 64 == 0) or the plain MFMA kernel.  fp32 mode: one thread per output.
// Returns true if the kernel left the per-tile LayerNorm statistics of its output in e.stats_out in the layout of the
// LDS-staged kernel (more than 16 rows, no split over K).
bool gemm(bpd_ctx* ctx, const GemmP& p, const Epi& e_in, int groups = 1) {
  hipStream_t s = ctx->stream;
  Epi e = e_in;
  if (ctx->cfg.dtype != BPD_BF16) {
    dim3 grid((p.N + 127) / 128, p.M, groups);
    hipLaunchKernelGGL(gemm_f32_kernel, grid, dim3(128), 0, s, p, e);
    return false;
  }
  LnP none{};
  if (stream_ok(ctx, p, e, groups)) {
    launch_stream(ctx, p, e, groups);
  } else if (skinny_ok(ctx, p)) {
    if (p.N / 16 >= 2048) launch_skinny<2, false, false>(ctx, p, e, none, nullptr, nullptr, groups);
    else launch_skinny<1, false, false>(ctx, p, e, none, nullptr, nullptr, groups);
  } else if (p.K % 64 == 0) {
    // In-place residual update with a long K and few output tiles: split K over workgroups.  The
    // slices are added, in a fixed order, by the LayerNorm kernel that reads the residual next.
    if (groups == 1 && e.mode == 0 && e.R && e.R == e.Yf && !e.Ya && !e.relu && !e.lnR_stats &&
        e.ldr == p.N && e.ldyf == p.N && p.N == ctx->cfg.d_model && p.K >= 2048) {
      const int ns = residual_k_slices(ctx, p);
      if (ns > 1) {
        GemmP q = p;
        q.ksplit = ns; q.part = ctx->lay.kpart;
        e.stats_out = nullptr;                     // the slices are raw products: no statistics of the sum yet
        dispatch_ldsx<false>(q, e, nullptr, nullptr, ns, s, ctx->lay.zeros);
        ctx->pend_slices = ns; ctx->pend_bias = e.bias ? e.bias : ctx->lay.zeros; ctx->pend_x = e.Yf;
        return false;
      }
    }
    return dispatch_ldsx<false>(p, e, nullptr, nullptr, groups, s, ctx->lay.zeros);
  } else {
    e.stats_out = nullptr;
    if (p.M > 64) launch_gemm_bf16<8, 1, 4>(p, e, groups, s);
    else launch_gemm_bf16<4, 1, 4>(p, e, groups, s);
  }
  return false;
}

void layernorm(bpd_ctx* ctx, float* x, LnW w, int M, void* ya, float* yf);

// Y = epilogue(LayerNorm(x) W).  Block of <= 16 rows: LayerNorm is applied inside the skinny
// kernel from the partial statistics the producer of x left in L.stats_ln.  More rows, with per-tile statistics of
// x in L.stats_big: applied while the LDS-staged kernel stages its activations (up to 128 rows) or folded into the
// weights (beyond).  Otherwise a LayerNorm kernel (into `xn`, and `yf` in fp32 if given) followed by the GEMM.
void gemm_ln(bpd_ctx* ctx, float* x, LnW w, void* xn, float* yf, GemmP p, const Epi& e, bool with_stats, bool big_stats = false,
             const FoldW* fold = nullptr) {
  // fold: the producer of x left its bf16 copy in xn and per-tile statistics in L.stats_big (more than 128 rows): one
  // GEMM on the weights with this LayerNorm folded in
  if (fold && fold->W && big_stats && !yf && ldsx_ln_ok(ctx, p)) {
    p.X = xn; p.W = fold->W;
    Epi ef = e;
    ef.ra_stats = ctx->lay.stats_big; ef.ra_c = fold->c; ef.ra_d = fold->d; ef.ra_eps = ctx->cfg.ln_eps;
    dispatch_ldsx_fold(p, ef, ctx->stream, ctx->lay.zeros);
    return;
  }
  // with_stats: the producer of x left its partial LayerNorm statistics in L.stats_ln (decoder block of one
  // row tile only; the encoder's kernels do not write them)
  if (with_stats && stats_path(ctx, p.M) && p.K == ctx->cfg.d_model) {
    LnP ln{x, w.g, w.b, ctx->lay.stats_ln, ctx->cfg.ln_eps};
    if (p.N / 16 >= 2048) launch_skinny<2, true, false>(ctx, p, e, ln, nullptr, nullptr, 1);
    else launch_skinny<1, true, false>(ctx, p, e, ln, nullptr, nullptr, 1);
    return;
  }
  // big_stats: more than 16 rows and the GEMM that produced x left per-tile statistics in L.stats_big
  if (big_stats && !yf && p.M <= LDSX_LN_M_MAX && ldsx_ln_ok(ctx, p)) {
    LnP ln{x, w.g, w.b, ctx->lay.stats_big, ctx->cfg.ln_eps};
    dispatch_ldsx_ln(p, e, ln, ctx->stream, ctx->lay.zeros);
    return;
  }
  layernorm(ctx, x, w, p.M, xn, yf);
  p.X = xn;
  gemm(ctx, p, e);
}

// Vocabulary projection with fused arg-max (bf16 mode).
// ---- streaming vocabulary projection: 17 .. 128 rows, K = 512 / 1024, at least one column tile per wave ----
size_t stream_vocab_lds_bytes(const GemmP& p) {
  const int rows = p.M < 64 ? p.M : 64;
  return (size_t)8 * 64 * 8 + (size_t)rows * (p.K + 8) * 2;
}
// workgroups per row block: one per CU of the row block's share, fewer when that leaves a wave less than two units of
// 16 weight loads to take turns with (K = 512: a unit is a whole column tile; 32000 columns at 64 rows: 14.5 us with
// 100 .. 167 workgroups, 15.5 us with 250, whose 250 atomics per row also cost more)
int stream_vocab_gx(const bpd_ctx* ctx, const GemmP& p) {
  const int rb = (p.M + 63) / 64, per = p.K == 512 ? 12 : 8;      // column tiles per workgroup, at least
  int gx = ctx->num_cus / rb;
  if (gx > p.N / 16 / per) gx = p.N / 16 / per;
  return gx < 1 ? 1 : gx;
}
bool stream_vocab_ok(const bpd_ctx* ctx, const GemmP& p) {
  const int rb = (p.M + 63) / 64;
  return ctx->cfg.dtype == BPD_BF16 && p.M > 16 && p.M <= 128 && (p.K == 512 || p.K == 1024) && p.N % 16 == 0 &&
         p.ldx % 8 == 0 && 2 * rb * stream_vocab_gx(ctx, p) >= ctx->num_cus &&       // at least half the chip streams
         stream_vocab_lds_bytes(p) <= (size_t)160 * 1024;
}
template <int NT, int UPT>
void launch_stream_vocab_cfg(const bpd_ctx* ctx, const GemmP& p, unsigned long long* keys, float* logits) {
  const size_t lds = stream_vocab_lds_bytes(p);
  auto k = stream_vocab_kernel<4, NT, UPT, false>;
  static size_t attr = 0;                       // per instantiation: allow more than 64 KiB of LDS
  if (attr < lds) { (void)hipFuncSetAttribute((const void*)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds); attr = lds; }
  hipLaunchKernelGGL(k, dim3(stream_vocab_gx(ctx, p), (p.M + 63) / 64), dim3(512), lds, ctx->stream, p, keys, logits);
}
void launch_stream_vocab(const bpd_ctx* ctx, const GemmP& p, unsigned long long* keys, float* logits) {
  // one column tile at a time.  Two at a time (NT = 2: one LDS read feeds two MFMAs) measured slower, 20.2 vs 18.5 us at
  // 100 x 1024 x 32768, and so did non-temporal loads (the second row block reads the same weights out of L2).
  if (p.K == 1024) launch_stream_vocab_cfg<1, 2>(ctx, p, keys, logits);
  else launch_stream_vocab_cfg<1, 1>(ctx, p, keys, logits);
}

void vocab_argmax(bpd_ctx* ctx, const GemmP& p, unsigned long long* keys, float* logits) {
  hipStream_t s = ctx->stream;
  Epi none{};
  LnP noln{};
  if (skinny_ok(ctx, p)) launch_skinny<2, false, true>(ctx, p, none, noln, keys, logits, 1);
  else if (stream_vocab_ok(ctx, p)) launch_stream_vocab(ctx, p, keys, logits);
  else if (p.K % 64 == 0) dispatch_ldsx<true>(p, none, keys, logits, 1, s);
  else {
    const int ntiles = p.N / 16;
    dim3 grid(ntiles, (p.M + 127) / 128, 1);
    hipLaunchKernelGGL((vocab_argmax_bf16_kernel<8, 1, 4>), grid, dim3(256), 0, s, p, keys, logits);
  }
}

GemmP gp(const void* X, int ldx, const void* W, int ldw, int M, int N, int K) {
  GemmP p{};
  p.X = X; p.ldx = ldx; p.W = W; p.ldw = ldw; p.M = M; p.N = N; p.K = K;
  return p;
}
Epi plain(const float* bias, int relu, const float* R, int ldr, float* Yf, int ldyf, void* Ya, int ldya) {
  Epi e{};
  e.mode = 0; e.bias = bias; e.relu = relu; e.R = R; e.ldr = ldr; e.Yf = Yf; e.ldyf = ldyf; e.Ya = Ya; e.ldya = ldya;
  return e;
}
Epi split(float* Qf, void* Ka, void* Va, int dsplit, int chunk0, int rows_per_seq, int cap, const int* base) {
  Epi e{};
  e.mode = 1; e.Qf = Qf; e.Ka = Ka; e.Va = Va; e.dsplit = dsplit; e.chunk0 = chunk0;
  e.rows_per_seq = rows_per_seq; e.cap = cap; e.base = base;
  return e;
}

void layernorm(bpd_ctx* ctx, float* x, LnW w, int M, void* ya, float* yf) {
  const int d = ctx->cfg.d_model;
  dim3 grid((M + 3) / 4);
  int nsl = 0;
  const float* bias = nullptr;
  if (ctx->pend_slices && ctx->pend_x == x) { nsl = ctx->pend_slices; bias = ctx->pend_bias; ctx->pend_slices = 0; }
#define BPD_LN(ACT_, V_) hipLaunchKernelGGL((layernorm_kernel<ACT_, V_>), grid, dim3(256), 0, ctx->stream, x, w.g, w.b, M, d, \
                                            ctx->cfg.ln_eps, (ACT_*)ya, yf, (const float*)ctx->lay.kpart, nsl, bias)
  if (ctx->cfg.dtype == BPD_BF16) {
    if (d <= 1024) BPD_LN(bf16_t, 4); else BPD_LN(bf16_t, LN_V);
  } else {
    if (d <= 1024) BPD_LN(float, 4); else BPD_LN(float, LN_V);
  }
#undef BPD_LN
}

// merge of the split attention's partial results: as few partials read per thread as the split needs
template <typename ACT, int DH>
void launch_combine(const AttnP& p, dim3 grid, hipStream_t s) {
  if (p.nsplit <= 4) hipLaunchKernelGGL((attention_combine_kernel<ACT, DH, 4>), grid, dim3(256), 0, s, p);
  else if (p.nsplit <= 8) hipLaunchKernelGGL((attention_combine_kernel<ACT, DH, 8>), grid, dim3(256), 0, s, p);
  else hipLaunchKernelGGL((attention_combine_kernel<ACT, DH, 16>), grid, dim3(256), 0, s, p);
}

int attention_nsplit(const bpd_ctx* ctx, int cap, int B, int R, int causal) {
  return attention_nsplit_of(ctx->cfg, (long)ctx->steps, ctx->local_q, ctx->local_m, cap, B, R, causal);
}

// Cross-attention whose query projection runs inside the attention kernel: LayerNorm statistics of x at hand (the
// caller checks), at most 16 rows per sequence, 64-wide heads, d = 128 / 256 / 512 / 1024, one workgroup per (head,
// sequence) and few enough of them that each streaming its head's 128 d bytes of weights beats one GEMM doing it once.
constexpr int ATTN_QPROJ_MAX_WGS = 128;       // (512 workgroups, batch 32 of Transformer-big: the step took 26 us longer than with the separate GEMM)
bool attention_qproj_ok(const bpd_ctx* ctx, int B, int R) {
  const bpd_config& c = ctx->cfg;
  const int d = c.d_model;
  return c.dtype == BPD_BF16 && R <= 16 && d == 64 * c.n_heads && (d == 128 || d == 256 || d == 512 || d == 1024) &&
         c.n_heads * B <= ATTN_QPROJ_MAX_WGS && attention_nsplit(ctx, c.max_src_len, B, R, 0) == 1;
}

void attention(bpd_ctx* ctx, const float* Q, const void* Kc, const void* Vc, void* out, int cap,
               int B, int R, const int* limit, int causal, const QProjP* qproj = nullptr) {
  const long kv_seq_stride = (long)cap * ctx->cfg.d_model;
  const bpd_config& c = ctx->cfg;
  const int dh = c.d_model / c.n_heads;
  AttnP p{};
  p.Q = Q; p.Kc = Kc; p.Vc = Vc; p.out = out; p.kv_seq_stride = kv_seq_stride; p.cap = cap; p.d = c.d_model; p.R = R;
  p.limit = limit; p.causal = causal; p.scale = 1.0f / sqrtf((float)dh);
  const bool local = causal && ctx->local_q > 0;
  p.local_q = local ? ctx->local_q : 0; p.local_m = local ? ctx->local_m : 0;
  const int tiles = (R + 15) / 16, wgs = c.n_heads * B * tiles;
  const int nsplit = attention_nsplit(ctx, cap, B, R, causal);
  p.nsplit = nsplit; p.part = ctx->lay.attn_part;
  dim3 grid(c.n_heads, B, tiles * nsplit), cgrid(c.n_heads, B, tiles);
  if (c.dtype == BPD_BF16) {
    if (dh == 64) {
      // a K/V buffer beyond half the last-level cache is streamed past it
      const size_t kv_bytes = (size_t)2 * c.n_dec_layers * B * cap * c.d_model * 2;
      // many workgroups: fetch only the rows in use (the length is read first); few: one round trip, rows past the end too
      // (a split launch walks a long cache, where nearly all fetched rows are in use: measured slower with the extra round trip)
      // (local attention: where the keys start depends on the length, so it is always read first)
      const bool limf = (nsplit == 1 && wgs >= ATTN_LIMF_MIN_WGS) || local;
      if (qproj) {                               // queries projected in the kernel (attention_qproj_ok() holds)
        switch (c.d_model / 128) {
          case 1: hipLaunchKernelGGL((attention_mfma_kernel<false, false, 1>), grid, dim3(256), 0, ctx->stream, p, *qproj); break;
          case 2: hipLaunchKernelGGL((attention_mfma_kernel<false, false, 2>), grid, dim3(256), 0, ctx->stream, p, *qproj); break;
          case 4: hipLaunchKernelGGL((attention_mfma_kernel<false, false, 4>), grid, dim3(256), 0, ctx->stream, p, *qproj); break;
          default: hipLaunchKernelGGL((attention_mfma_kernel<false, false, 8>), grid, dim3(256), 0, ctx->stream, p, *qproj); break;
        }
        return;
      }
      if (causal && kv_bytes > ((size_t)128 << 20)) {
        if (limf) hipLaunchKernelGGL((attention_mfma_kernel<true, true, 0>), grid, dim3(256), 0, ctx->stream, p, QProjP{});
        else hipLaunchKernelGGL((attention_mfma_kernel<true, false, 0>), grid, dim3(256), 0, ctx->stream, p, QProjP{});
      } else {
        if (limf) hipLaunchKernelGGL((attention_mfma_kernel<false, true, 0>), grid, dim3(256), 0, ctx->stream, p, QProjP{});
        else hipLaunchKernelGGL((attention_mfma_kernel<false, false, 0>), grid, dim3(256), 0, ctx->stream, p, QProjP{});
      }
      if (nsplit > 1) launch_combine<bf16_t, 64>(p, cgrid, ctx->stream);
    } else {
      hipLaunchKernelGGL((attention_kernel<bf16_t, 16>), grid, dim3(256), 0, ctx->stream, p);
      if (nsplit > 1) launch_combine<bf16_t, 16>(p, cgrid, ctx->stream);
    }
  } else {
    hipLaunchKernelGGL((attention_kernel<float, 16>), grid, dim3(256), 0, ctx->stream, p);
    if (nsplit > 1) launch_combine<float, 16>(p, cgrid, ctx->stream);
  }
}

void embed(bpd_ctx* ctx, const int* tok, int tok_ld, const int* base, int rows_per_seq, int M, const float* pos,
           float* x, int zero_input, unsigned long long* keys = nullptr, int nkeys = 0) {
  const bpd_config& c = ctx->cfg;
  const long n = (long)M * c.d_model;
  dim3 grid((unsigned)((n + 255) / 256));
  const float scale = sqrtf((float)c.d_model);
  if (stats_path(ctx, M) && x == ctx->lay.x) {
    hipLaunchKernelGGL(embed_stats_kernel, dim3(c.d_model / 16), dim3(64), 0, ctx->stream, tok, tok_ld, base, rows_per_seq, M,
                       c.d_model, (const bf16_t*)ctx->lay.emb, c.vocab, pos, scale, x, zero_input, ctx->lay.stats_ln, keys, nkeys);
    return;
  }
  if (c.dtype == BPD_BF16)
    hipLaunchKernelGGL(embed_kernel<true>, grid, dim3(256), 0, ctx->stream, tok, tok_ld, base, rows_per_seq, M, c.d_model,
                       ctx->lay.emb, c.vocab, pos, scale, x, zero_input, keys, nkeys);
  else
    hipLaunchKernelGGL(embed_kernel<false>, grid, dim3(256), 0, ctx->stream, tok, tok_ld, base, rows_per_seq, M, c.d_model,
                       ctx->lay.emb, c.vocab, pos, scale, x, zero_input, keys, nkeys);
}

void fill_i32(bpd_ctx* ctx, int* p, long n, int v) {
  hipLaunchKernelGGL(fill_i32_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, ctx->stream, p, n, v);
}

// ------------------------------------------------------------------------------- decoder stack kernel
// The decoder layers of a block of at most 16 rows as one kernel on one XCD (bpd_stack.h).  Usable when the workgroup
// placement probe of bpd_create found the regular round-robin, the model has a shape the kernel is built for, both
// attentions run unsplit (short caches), and the largest operator's LDS fits.
StackShape stack_shape_of(const bpd_ctx* ctx, int B, int R) {
  const bpd_config& c = ctx->cfg;
  StackShape s;
  s.n_layers = c.n_dec_layers; s.d = c.d_model; s.F = c.d_ff; s.heads = c.n_heads; s.B = B; s.M = B * R;
  s.workers = ctx->stack_workers; s.KU = c.d_model / 128;
  return s;
}
int stack_lds_bytes(const bpd_ctx* ctx, int B, int R) { return stack_lds_need(stack_shape_of(ctx, B, R), (int)AttnLds::BYTES); }
bool stack_usable(const bpd_ctx* ctx, int B, int R) {
  const bpd_config& c = ctx->cfg;
  const int M = B * R;
  return ctx->stack_workers > 0 && !ctx->stack_off && ctx->lay.stack_ex != nullptr && M >= 1 && M <= 16 && ctx->local_q == 0 &&
         attention_nsplit(ctx, c.max_out_len + c.k_max + 1, B, R, 1) == 1 && attention_nsplit(ctx, c.max_src_len, B, R, 0) == 1 &&
         stack_lds_bytes(ctx, B, R) <= 160 * 1024 &&
         (std::max(3 * c.d_model, c.d_ff) / 16 + ctx->stack_workers - 1) / ctx->stack_workers <= 8;     // tiles a helper wave finishes: two
}
template <int KU>
void launch_stack_ku(bpd_ctx* ctx, const StackP& p) {
  auto k = decoder_stack_kernel<KU>;
  static int attr = 0;                            // per instantiation: allow more than 64 KiB of LDS
  if (attr < p.lds_bytes) { (void)hipFuncSetAttribute((const void*)k, hipFuncAttributeMaxDynamicSharedMemorySize, p.lds_bytes); attr = p.lds_bytes; }
  hipLaunchKernelGGL(k, dim3(p.nx * p.workers), dim3(512), p.lds_bytes, ctx->stream, p);
}
void launch_stack(bpd_ctx* ctx, int R) {
  const bpd_config& c = ctx->cfg;
  Layout& L = ctx->lay;
  const int d = c.d_model, slots = c.max_out_len + c.k_max + 1;
  StackP p{};
  p.L = (const StackLayerP*)L.stack_layers;
  p.n_layers = c.n_dec_layers; p.d = d; p.F = c.d_ff; p.heads = c.n_heads; p.B = ctx->B; p.R = R; p.M = ctx->B * R;
  p.slots = slots; p.max_src = c.max_src_len;
  p.Lbase = L.L; p.src_len = L.src_len; p.x_in = L.x; p.x_out = L.x; p.stats_out = L.stats_ln;
  p.ex = L.stack_ex; p.flags = L.stack_flags; p.err = L.stack_err;
  if (++ctx->stack_epoch == 0) ctx->stack_epoch = 1;
  p.epoch = ctx->stack_epoch;
  p.spin_limit = 1 << 21;
  p.xcc = ctx->stack_xcc; p.nx = ctx->stack_nx; p.workers = ctx->stack_workers;
  p.eps = c.ln_eps; p.scale = 1.0f / sqrtf(64.f);
  p.lds_bytes = stack_lds_bytes(ctx, ctx->B, R);
  p.trace = getenv("BPD_STACK_TRACE") ? L.stack_trace : nullptr;
  switch (d / 128) {
    case 1: launch_stack_ku<1>(ctx, p); break;
    case 2: launch_stack_ku<2>(ctx, p); break;
    case 4: launch_stack_ku<4>(ctx, p); break;
    case 6: launch_stack_ku<6>(ctx, p); break;
    default: launch_stack_ku<8>(ctx, p); break;
  }
}
// After a synchronisation: has a stack launch reported a wait that ran out?  Then the per-operator kernels take over
// for the rest of the context's life and the caller learns that results since the last check cannot be trusted.
int stack_check(bpd_ctx* ctx) {
  if (ctx->stack_workers == 0 || ctx->stack_off || ctx->stack_epoch == 0) return BPD_OK;
  unsigned e = 0;
  HIPCHK(hipMemcpy(&e, ctx->lay.stack_err, 4, hipMemcpyDeviceToHost));
  if (e == 0) return BPD_OK;
  ctx->stack_off = true;
  HIPCHK(hipMemsetAsync(ctx->lay.stack_err, 0, 4, ctx->stream));
  return fail(ctx, BPD_E_HIP, "decoder stack kernel: a bounded wait ran out (code " + std::to_string(e) +
                              "); the results of this decode are invalid, later steps use the per-operator kernels");
}

// ------------------------------------------------------------------------------- profiling

hipEvent_t prof_event(bpd_ctx* ctx) {
  if (ctx->prof_used == ctx->prof_ev.size()) {
    hipEvent_t e;
    (void)hipEventCreate(&e);
    ctx->prof_ev.push_back(e);
  }
  return ctx->prof_ev[ctx->prof_used++];
}
struct PhaseTimer {
  bpd_ctx* ctx; bool on;
  PhaseTimer(bpd_ctx* c, int phase) : ctx(c), on(c->prof_phase == phase) {
    if (on) (void)hipEventRecord(prof_event(ctx), ctx->stream);
  }
  ~PhaseTimer() {
    if (on) { (void)hipEventRecord(prof_event(ctx), ctx->stream); ctx->prof_launches++; }
  }
};

// ------------------------------------------------------------------------------- the model invocation

StateP state_params(bpd_ctx* ctx);

// Heads and vocabulary projection of one step in two dependent phases (same tokens as the k x k
// table, fewer rows): p_1 at the k block rows -> verify -> the heads 2..k at row k-hat only, which
// is all the accept and predict substeps read (Section 3: verification uses p_1, the next
// proposals are row k-hat of the table).  2k - 1 rows of the vocabulary projection per sequence
// instead of k^2.  Needs more than 16 block rows (the single-tile path keeps its fused LayerNorm).
int heads_two_phase(bpd_ctx* ctx, int k) {
  const bpd_config& c = ctx->cfg;
  Layout& L = ctx->lay;
  const int B = ctx->B, d = c.d_model, F = c.d_ff, M = B * k;
  const size_t as = act_size(c);
  // phase 1: head 1 (the base model's p_1) at every block row
  layernorm(ctx, L.x, L.dec_lnf, M, L.hn, L.h);
  gemm(ctx, gp(L.hn, d, L.hw1, c.k_max * F, M, F, d), plain(L.hb1, 1, nullptr, 0, nullptr, 0, L.H, F));
  gemm(ctx, gp(L.H, F, L.hw2, d, M, d, F), plain(L.hb2, 0, L.h, d, nullptr, 0, L.O, d));
  unsigned long long* keys2 = L.keys_h1 + M;           // this step's second-phase keys follow its M head-1 keys: one fill clears both
  fill_i32(ctx, (int*)L.keys_h1, 4L * M, 0);
  const bool topn = ctx->top_n > 1;
  vocab_argmax(ctx, gp(L.O, d, L.emb, c.vocab, M, c.vocab, d), L.keys_h1, topn ? L.logits_h1 : nullptr);
  if (topn)
    hipLaunchKernelGGL(topn_rank_kernel, dim3(k - 1, B), dim3(256), 0, ctx->stream, (const float*)L.logits_h1, c.vocab,
                       (const int*)L.P, c.k_max, k, ctx->top_n, L.topn_ok);
  StateP st = state_params(ctx);
  st.imposed = ctx->cur_imposed; st.imposed_stride = ctx->cur_imposed_stride;
  hipLaunchKernelGGL(select_row_kernel, dim3(B), dim3(256), 0, ctx->stream, st, (const unsigned long long*)L.keys_h1, k,
                     ctx->cur_imposed_step, (const bf16_t*)L.hn, (const float*)L.h, d, L.sel, (bf16_t*)L.hn2, L.h2);
  // phase 2: heads 2..k at the selected row of each sequence
  const int kh = k - 1;
  const char* w1 = (const char*)L.hw1 + (size_t)F * d * as;          // packed by 16-column tiles: head 2 starts F columns in
  const char* w2 = (const char*)L.hw2 + (size_t)F * d * as;
  gemm(ctx, gp(L.hn2, d, w1, c.k_max * F, B, kh * F, d), plain(L.hb1 + F, 1, nullptr, 0, nullptr, 0, L.H, kh * F));
  {
    GemmP p = gp(L.H, kh * F, w2, d, B, d, F);
    p.x_g = F; p.w_g = (long)F * d;
    Epi e = plain(L.hb2 + d, 0, L.h2, d, nullptr, 0, L.O, kh * d);
    e.bias_g = d; e.r_g = 0; e.ya_g = d;
    gemm(ctx, p, e, kh);
  }
  vocab_argmax(ctx, gp(L.O, d, L.emb, c.vocab, B * kh, c.vocab, d), keys2, nullptr);
  hipLaunchKernelGGL(assemble_keys_kernel, dim3(B), dim3(256), 0, ctx->stream, (const unsigned long long*)L.keys_h1,
                     (const unsigned long long*)keys2, (const int*)L.sel, k, L.keys);
  LAUNCHCHK();
  if (ctx->pend_slices) return fail(ctx, BPD_E_STATE, "split-K slices were left unreduced");
  return BPD_OK;
}

// The folded copies of the decoder's LayerNorm + GEMM pairs follow the loaded weights: bpd_load_weights marks them stale
// (and asks for a new bpd_encode, which calls this).
void refresh_folded_weights(bpd_ctx* ctx) {
  Layout& L = ctx->lay;
  if (ctx->fold_ready || !L.dec[0].f_qkv.W) return;
  const bpd_config& c = ctx->cfg;
  const int d = c.d_model;
  auto fold = [&](const void* W, const FoldW& f, const LnW& w, int N) {
    hipLaunchKernelGGL(fold_layernorm_kernel, dim3(N / 16), dim3(64), 0, ctx->stream, (const bf16_t*)W, (bf16_t*)f.W, w.g, w.b, f.c, f.d, d / 32);
  };
  for (auto& e : L.dec) { fold(e.wqkv, e.f_qkv, e.ln1, 3 * d); fold(e.cq, e.f_cq, e.ln2, d); fold(e.w1, e.f_w1, e.ln3, c.d_ff); }
  ctx->fold_ready = true;
}

// One invocation of the combined model on R new rows per sequence (R = 1 for the first call
// on the empty prefix, R = k afterwards) with the first k heads; fills keys[B*R*k].
int forward(bpd_ctx* ctx, int R, int k, int zero_input, float* logits) {
  const bpd_config& c = ctx->cfg;
  Layout& L = ctx->lay;
  const int B = ctx->B, d = c.d_model, F = c.d_ff, M = B * R;
  const int slots = c.max_out_len + c.k_max + 1;
  const size_t as = act_size(c);
  const long nk = (long)M * k;
  const bool sp = stats_path(ctx, M);
  // residual update x += ...; on the statistics path the kernel also leaves LayerNorm partial sums
  // with more rows the LDS-staged kernel leaves them per tile in L.stats_big for the LayerNorm-fused GEMM that follows
  // (up to 128 rows: with more, every column block repeating the normalisation of its rows costs more than the kernel saved)
  const bool bigs = !sp && c.dtype == BPD_BF16 && M > 16 && M <= LDSX_LN_M_MAX && d % 64 == 0 && d <= 1024;
  // more than 128 rows: the GEMMs that update x also leave its bf16 copy in L.xn, and the LayerNorm + GEMM that follows
  // runs as one GEMM on folded weights (unless that update is split over K: its slices are summed by a LayerNorm kernel)
  const bool folds = !sp && !bigs && c.dtype == BPD_BF16 && M > LDSX_LN_M_MAX && L.dec[0].f_qkv.W != nullptr;
  auto residual = [&](const float* bias, int K) {
    Epi e = plain(bias, 0, L.x, d, L.x, d, nullptr, 0);
    if (sp) e.stats_out = L.stats_ln;
    else if (bigs) e.stats_out = L.stats_big;
    else if (folds && residual_k_slices(ctx, gp(nullptr, K, nullptr, d, M, d, K)) == 1) { e.stats_out = L.stats_big; e.Ya = L.xn; e.ldya = d; }
    return e;
  };
  bool xs = false;      // L.stats_big describes the current L.x
  {
    PhaseTimer t(ctx, BPD_PHASE_LAYERS);
    // (the previous step's accept kernel may already have embedded this block, with its statistics (and, beyond 16 rows,
    // its bf16 copy in L.xn), and cleared the keys)
    const bool have_x = embed_in_accept(ctx) && !zero_input && R == k && ctx->x_ready_k == k;
    ctx->x_ready_k = 0;
    xs = have_x && !sp;
    if (!have_x) embed(ctx, L.P, c.k_max, L.L, R, M, L.pos_tgt, L.x, zero_input, L.keys, (int)nk);
    const bool stack = sp && stack_usable(ctx, B, R);
    if (stack) launch_stack(ctx, R);
    for (int l = 0; l < (stack ? 0 : c.n_dec_layers); ++l) {
      DecL& w = L.dec[l];
      char* Kl = (char*)L.selfK + (size_t)l * c.max_batch * slots * d * as;
      char* Vl = (char*)L.selfV + (size_t)l * c.max_batch * slots * d * as;
      char* cK = (char*)L.crossK + (size_t)l * c.max_batch * c.max_src_len * d * as;
      char* cV = (char*)L.crossV + (size_t)l * c.max_batch * c.max_src_len * d * as;
      // self-attention sublayer: K/V of the block rows go straight into the cache at L_b + i'
      gemm_ln(ctx, L.x, w.ln1, L.xn, nullptr, gp(L.xn, d, w.wqkv, 3 * d, M, 3 * d, d), split(L.q, Kl, Vl, d, 0, R, slots, L.L), sp, xs, folds ? &w.f_qkv : nullptr);
      attention(ctx, L.q, Kl, Vl, L.attn, slots, B, R, L.L, 1);
      xs = gemm(ctx, gp(L.attn, d, w.wo, d, M, d, d), residual(nullptr, d));
      // cross-attention sublayer over the encoder memory
      if ((sp || xs) && attention_qproj_ok(ctx, B, R)) {
        const QProjP qp{L.x, w.ln2.g, w.ln2.b, sp ? L.stats_ln : L.stats_big, sp ? 16 : M, w.cq, c.ln_eps};
        attention(ctx, nullptr, cK, cV, L.attn, c.max_src_len, B, R, L.src_len, 0, &qp);
      } else {
        gemm_ln(ctx, L.x, w.ln2, L.xn, nullptr, gp(L.xn, d, w.cq, d, M, d, d), plain(nullptr, 0, nullptr, 0, L.q, d, nullptr, 0), sp, xs, folds ? &w.f_cq : nullptr);
        attention(ctx, L.q, cK, cV, L.attn, c.max_src_len, B, R, L.src_len, 0);
      }
      xs = gemm(ctx, gp(L.attn, d, w.co, d, M, d, d), residual(nullptr, d));
      // feed-forward sublayer
      gemm_ln(ctx, L.x, w.ln3, L.xn, nullptr, gp(L.xn, d, w.w1, F, M, F, d), plain(w.b1, 1, nullptr, 0, nullptr, 0, L.ffh, F), sp, xs, folds ? &w.f_w1 : nullptr);
      xs = gemm(ctx, gp(L.ffh, F, w.w2, d, M, d, F), residual(w.b2, F));
    }
  }
  { PhaseTimer t(ctx, BPD_PHASE_EMPTY); }       // calibration of the event bracketing itself
  if (ctx->two_phase && R == k && k > 1 && M > 16 && !logits && c.dtype == BPD_BF16) return heads_two_phase(ctx, k);
  // the k residual FFN heads: final LayerNorm + hidden layers side by side (h kept in fp32
  // for the residual), then one output layer per head
  {
    PhaseTimer t(ctx, BPD_PHASE_HEAD_HIDDEN);
    gemm_ln(ctx, L.x, L.dec_lnf, L.hn, L.h, gp(L.hn, d, L.hw1, c.k_max * F, M, k * F, d),
            plain(L.hb1, 1, nullptr, 0, nullptr, 0, L.H, k * F), sp);
  }
  {
    PhaseTimer t(ctx, BPD_PHASE_HEAD_OUT);
    GemmP p = gp(L.H, k * F, L.hw2, d, M, d, F);
    p.x_g = F; p.w_g = (long)F * d;
    Epi e = plain(L.hb2, 0, L.h, d, nullptr, 0, L.O, k * d);
    e.bias_g = d; e.r_g = 0; e.ya_g = d;
    if (sp) {          // h = LayerNorm(x) is recomputed from x and the partial statistics
      e.R = L.x; e.lnR_stats = L.stats_ln; e.lnR_g = L.dec_lnf.g; e.lnR_b = L.dec_lnf.b; e.lnR_K = d; e.lnR_eps = c.ln_eps;
    }
    gemm(ctx, p, e, k);
  }
  {
    PhaseTimer t(ctx, BPD_PHASE_VOCAB);
    if (c.dtype == BPD_BF16) {
      vocab_argmax(ctx, gp(L.O, d, L.emb, c.vocab, (int)nk, c.vocab, d), L.keys, logits);
    } else {
      hipLaunchKernelGGL(vocab_argmax_f32_kernel, dim3((unsigned)nk), dim3(256), 0, ctx->stream, (const float*)L.O, d,
                         (const float*)L.emb, (int)nk, c.vocab, d, L.keys, logits);
    }
    // top-n acceptance: p_1 of every block row once more with its logits kept (rows of head 1 are
    // every k-th row of O), then the rank of each proposal among them
    if (ctx->top_n > 1 && R == k && k > 1) {
      fill_i32(ctx, (int*)L.keys_h1, 2L * M, 0);
      if (c.dtype == BPD_BF16) {
        vocab_argmax(ctx, gp(L.O, k * d, L.emb, c.vocab, M, c.vocab, d), L.keys_h1, L.logits_h1);
      } else {
        hipLaunchKernelGGL(vocab_argmax_f32_kernel, dim3((unsigned)M), dim3(256), 0, ctx->stream, (const float*)L.O, k * d,
                           (const float*)L.emb, M, c.vocab, d, L.keys_h1, L.logits_h1);
      }
      hipLaunchKernelGGL(topn_rank_kernel, dim3(k - 1, B), dim3(256), 0, ctx->stream, (const float*)L.logits_h1, c.vocab,
                         (const int*)L.P, c.k_max, k, ctx->top_n, L.topn_ok);
    }
  }
  LAUNCHCHK();
  if (ctx->pend_slices) return fail(ctx, BPD_E_STATE, "split-K slices were left unreduced");
  return BPD_OK;
}

StateP state_params(bpd_ctx* ctx) {
  Layout& L = ctx->lay;
  StateP s{};
  s.L = L.L; s.j = L.j; s.finished = L.finished; s.max_len = L.max_len; s.P = L.P; s.A = L.A;
  s.accepted = L.accepted; s.out_ids = L.out_ids; s.stats = L.stats; s.imposed = nullptr; s.imposed_stride = 0;
  s.kmax = ctx->cfg.k_max; s.max_out = ctx->cfg.max_out_len;
  s.eos_id = ctx->cfg.eos_id; s.distance_eps = ctx->distance_eps; s.min_block = ctx->min_block;
  s.topn_ok = ctx->top_n > 1 ? ctx->lay.topn_ok : nullptr;
  return s;
}

int encoder(bpd_ctx* ctx) {
  const bpd_config& c = ctx->cfg;
  Layout& L = ctx->lay;
  const int B = ctx->B, S = ctx->S, d = c.d_model, F = c.d_ff, M = B * S;
  const size_t as = act_size(c);
  embed(ctx, L.src_ids, S, nullptr, S, M, L.pos_src, L.xe, 0);
  // 17 .. 128 source rows: the residual GEMMs leave LayerNorm statistics for the LayerNorm-fused GEMM that follows
  const bool bigs = c.dtype == BPD_BF16 && M > 16 && M <= LDSX_LN_M_MAX && d % 64 == 0 && d <= 1024;
  auto residual = [&](const float* bias) {
    Epi e = plain(bias, 0, L.xe, d, L.xe, d, nullptr, 0);
    if (bigs) e.stats_out = L.stats_big;
    return e;
  };
  bool xs = false;      // L.stats_big describes the current L.xe
  for (int l = 0; l < c.n_enc_layers; ++l) {
    EncL& w = L.enc[l];
    gemm_ln(ctx, L.xe, w.ln1, L.xen, nullptr, gp(L.xen, d, w.wqkv, 3 * d, M, 3 * d, d), split(L.qe, L.ke, L.ve, d, 0, S, S, nullptr), false, xs);
    attention(ctx, L.qe, L.ke, L.ve, L.attne, S, B, S, L.src_len, 0);
    xs = gemm(ctx, gp(L.attne, d, w.wo, d, M, d, d), residual(nullptr));
    gemm_ln(ctx, L.xe, w.ln2, L.xen, nullptr, gp(L.xen, d, w.w1, F, M, F, d), plain(w.b1, 1, nullptr, 0, nullptr, 0, L.ffhe, F), false, xs);
    xs = gemm(ctx, gp(L.ffhe, F, w.w2, d, M, d, F), residual(w.b2));
  }
  layernorm(ctx, L.xe, L.enc_lnf, M, L.mem, nullptr);
  for (int l = 0; l < c.n_dec_layers; ++l) {
    char* cK = (char*)L.crossK + (size_t)l * c.max_batch * c.max_src_len * d * as;
    char* cV = (char*)L.crossV + (size_t)l * c.max_batch * c.max_src_len * d * as;
    gemm(ctx, gp(L.mem, d, L.dec[l].ckv, 2 * d, M, 2 * d, d), split(nullptr, cK, cV, d, 1, S, c.max_src_len, nullptr));
  }
  LAUNCHCHK();
  return BPD_OK;
}

__global__ void sanitize_kernel(int* src_len, int* max_len, int* src_ids, int B, int S, int max_out, int V) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < B) {
    int s = src_len[i]; src_len[i] = s < 1 ? 1 : (s > S ? S : s);
    int m = max_len[i]; max_len[i] = m < 1 ? 1 : (m > max_out ? max_out : m);
  }
  if (i < B * S) { int t = src_ids[i]; src_ids[i] = t < 0 ? 0 : (t >= V ? V - 1 : t); }
}

bool is_host_ptr(const void* p) {
  hipPointerAttribute_t a;
  if (hipPointerGetAttributes(&a, p) != hipSuccess) { (void)hipGetLastError(); return true; }
  return a.type != hipMemoryTypeDevice && a.type != hipMemoryTypeManaged;
}

// is_host_ptr with the answers for the last four distinct pointers remembered in the context
bool is_host_ptr_cached(bpd_ctx* ctx, const void* p) {
  for (int i = 0; i < 4; ++i)
    if (ctx->kind_ptr[i] == p) return ctx->kind_host[i];
  const bool h = is_host_ptr(p);
  ctx->kind_ptr[ctx->kind_next] = p; ctx->kind_host[ctx->kind_next] = h;
  ctx->kind_next = (ctx->kind_next + 1) & 3;
  return h;
}

}  // namespace

// ------------------------------------------------------------------------------- C ABI

extern "C" {

size_t bpd_workspace_bytes(const bpd_config* cfg) {
  if (!cfg || !config_ok(*cfg)) return 0;
  Layout L;
  return build_layout(*cfg, nullptr, L);
}

int bpd_create(const bpd_config* cfg, void* workspace, size_t workspace_bytes, void* hip_stream, bpd_ctx** out) {
  if (!cfg || !workspace || !out) return BPD_E_ARG;
  if (!config_ok(*cfg)) return BPD_E_ARG;
  if (((uintptr_t)workspace) % ALIGN) return BPD_E_ARG;
  Layout probe;
  if (workspace_bytes < build_layout(*cfg, nullptr, probe)) return BPD_E_CAPACITY;
  bpd_ctx* ctx = new bpd_ctx();
  ctx->cfg = *cfg;
  ctx->stream = (hipStream_t)hip_stream;
  {
    int dev = 0, cus = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) { delete ctx; return BPD_E_HIP; }
    ctx->device = dev;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess && cus > 0) ctx->num_cus = cus;
    if (!g_scratch_ptr[dev]) {               // once per device, with that device current
      void* sp = nullptr;
      if (hipGetSymbolAddress(&sp, HIP_SYMBOL(scratch)) != hipSuccess || !sp) { (void)hipGetLastError(); delete ctx; return BPD_E_HIP; }
      g_scratch_ptr[dev] = sp;
    }
  }
  build_layout(*cfg, (char*)workspace, ctx->lay);
  build_table(ctx);
  {
    const size_t d = cfg->d_model, F = cfg->d_ff, V = cfg->vocab, k = cfg->k_max;
    const size_t step_weights = ((size_t)cfg->n_dec_layers * (6 * d * d + 2 * d * F) + 2 * k * d * F + V * d) * act_size(*cfg);
    ctx->weights_exceed_llc = step_weights > ((size_t)192 << 20);
  }
  (void)hipMemsetAsync(ctx->lay.stack_err, 0, 256, ctx->stream);
  if (ctx->lay.stack_ex && ctx->num_cus <= XCC_MAP_MAX) {
    // placement probe: which XCD does workgroup i of a one-workgroup-per-CU grid land on?  The stack kernel needs the
    // regular round-robin (workgroup i on XCD i mod nx, every XCD equally often) and at most 64 workers per XCD.
    const char* env = getenv("BPD_DECODER_STACK");
    std::vector<StackLayerP> table(STACK_MAX_LAYERS);        // the layers' weights and caches: fixed addresses in the workspace
    {
      const bpd_config& c = *cfg;
      Layout& L = ctx->lay;
      const size_t d = c.d_model, slots = (size_t)c.max_out_len + c.k_max + 1, as = 2;
      for (int l = 0; l < c.n_dec_layers; ++l) {
        const DecL& w = L.dec[l];
        StackLayerP& q = table[l];
        q.wqkv = w.wqkv; q.wo = w.wo; q.cq = w.cq; q.co = w.co; q.w1 = w.w1; q.w2 = w.w2;
        q.ln1g = w.ln1.g; q.ln1b = w.ln1.b; q.ln2g = w.ln2.g; q.ln2b = w.ln2.b; q.ln3g = w.ln3.g; q.ln3b = w.ln3.b;
        q.b1 = w.b1; q.b2 = w.b2;
        q.selfK = (char*)L.selfK + (size_t)l * c.max_batch * slots * d * as;
        q.selfV = (char*)L.selfV + (size_t)l * c.max_batch * slots * d * as;
        q.crossK = (char*)L.crossK + (size_t)l * c.max_batch * c.max_src_len * d * as;
        q.crossV = (char*)L.crossV + (size_t)l * c.max_batch * c.max_src_len * d * as;
      }
      (void)hipMemcpyAsync(ctx->lay.stack_layers, table.data(), sizeof(StackLayerP) * STACK_MAX_LAYERS, hipMemcpyHostToDevice, ctx->stream);
    }
    (void)hipMemsetAsync(ctx->lay.stack_flags, 0, (size_t)cfg->n_dec_layers * STACK_OPS * STACK_FLAG_STRIDE * 4, ctx->stream);
    hipLaunchKernelGGL(xcc_map_kernel, dim3(ctx->num_cus), dim3(64), 0, ctx->stream, ctx->lay.xcc_map);
    std::vector<unsigned> map(ctx->num_cus);
    if (hipMemcpyAsync(map.data(), ctx->lay.xcc_map, map.size() * 4, hipMemcpyDeviceToHost, ctx->stream) == hipSuccess &&
        hipStreamSynchronize(ctx->stream) == hipSuccess && env && env[0] == '1') {      // opt-in: slower than the kernel chain so far
      int nx = 1;
      while (nx < ctx->num_cus && map[nx] != map[0]) ++nx;
      bool ok = ctx->num_cus % nx == 0 && ctx->num_cus / nx <= STACK_FLAG_STRIDE;
      for (int i = 0; ok && i < ctx->num_cus; ++i) ok = map[i] == map[i % nx];
      for (int i = 0; ok && i < nx; ++i)
        for (int j = 0; ok && j < i; ++j) ok = map[i] != map[j];
      if (ok) { ctx->stack_nx = nx; ctx->stack_xcc = (int)map[0]; ctx->stack_workers = ctx->num_cus / nx; }
    }
    (void)hipGetLastError();
  }
  (void)hipMemsetAsync(ctx->lay.zeros, 0, ctx->lay.n_zeros * 4, ctx->stream);
  (void)hipMemsetAsync(ctx->lay.stats_ln, 0, 64 * 16 * 2 * 4, ctx->stream);
  if (hipHostMalloc((void**)&ctx->pinned, 64 * sizeof(int), hipHostMallocDefault) != hipSuccess) {
    delete ctx;
    return BPD_E_HIP;
  }
  *out = ctx;
  return BPD_OK;
}

int bpd_destroy(bpd_ctx* ctx) {
  if (!ctx) return BPD_E_ARG;
  (void)hipStreamSynchronize(ctx->stream);
  if (const char* path = getenv("BPD_STACK_TRACE")) {      // debugging aid: the last stack launch's timestamps, raw
    if (ctx->lay.stack_trace && ctx->stack_workers > 0) {
      const size_t n = (size_t)ctx->stack_workers * ctx->cfg.n_dec_layers * STACK_OPS * 8;
      std::vector<unsigned long long> t(n);
      if (hipMemcpy(t.data(), ctx->lay.stack_trace, n * 8, hipMemcpyDeviceToHost) == hipSuccess)
        if (FILE* f = fopen(path, "wb")) { fwrite(t.data(), 8, n, f); fclose(f); }
    }
  }
  for (auto e : ctx->prof_ev) (void)hipEventDestroy(e);
  if (ctx->pinned) (void)hipHostFree(ctx->pinned);
  delete ctx;
  return BPD_OK;
}

const char* bpd_last_error(const bpd_ctx* ctx) { return ctx ? ctx->err.c_str() : "null context"; }

int bpd_load_weights(bpd_ctx* ctx, const bpd_tensor* tensors, int n) {
  if (!ctx || !tensors || n < 0) return fail(ctx, BPD_E_ARG, "bpd_load_weights: null argument");
  const bool bf = ctx->cfg.dtype == BPD_BF16;
  // validate everything first so that a bad tensor leaves the loaded set unchanged
  for (int t = 0; t < n; ++t) {
    const bpd_tensor& T = tensors[t];
    if (!T.name || !T.data) return fail(ctx, BPD_E_ARG, "bpd_load_weights: tensor without name or data");
    auto it = ctx->table.find(T.name);
    if (it == ctx->table.end()) return fail(ctx, BPD_E_WEIGHTS, std::string("unknown tensor ") + T.name);
    const WEntry& e = it->second;
    if (T.dtype != BPD_F32 && T.dtype != BPD_BF16) return fail(ctx, BPD_E_WEIGHTS, std::string("bad dtype for ") + T.name);
    bool ok = T.ndim == e.nd;
    for (int i = 0; ok && i < e.nd; ++i) ok = T.shape[i] == e.shape[i];
    if (!ok) return fail(ctx, BPD_E_WEIGHTS, std::string("wrong shape for ") + T.name);
    size_t count = 1;
    for (int i = 0; i < e.nd; ++i) count *= (size_t)e.shape[i];
    if (!T.on_device && count * (T.dtype == BPD_F32 ? 4 : 2) > ctx->lay.staging_bytes)
      return fail(ctx, BPD_E_CAPACITY, std::string("staging area too small for ") + T.name);
  }
  for (int t = 0; t < n; ++t) {
    const bpd_tensor& T = tensors[t];
    WEntry& e = ctx->table[T.name];
    size_t count = 1;
    for (int i = 0; i < e.nd; ++i) count *= (size_t)e.shape[i];
    const size_t esz = T.dtype == BPD_F32 ? 4 : 2;
    const void* src = T.data;
    if (!T.on_device) {                          // (fits the staging area: checked above)
      HIPCHK(hipMemcpyAsync(ctx->lay.staging, T.data, count * esz, hipMemcpyHostToDevice, ctx->stream));
      src = ctx->lay.staging;
    }
    const dim3 blk(256);
    auto conv_mat = [&](const void* s, void* dst, int K, int N, int transposed, int ldw, int n_off) {
      const long tot = (long)K * N;
      dim3 grid((unsigned)((tot + 255) / 256));
      if (T.dtype == BPD_F32) {
        if (bf) hipLaunchKernelGGL((convert_matrix_kernel<float, true>), grid, blk, 0, ctx->stream, (const float*)s, dst, K, N, transposed, ldw, n_off);
        else hipLaunchKernelGGL((convert_matrix_kernel<float, false>), grid, blk, 0, ctx->stream, (const float*)s, dst, K, N, transposed, ldw, n_off);
      } else {
        if (bf) hipLaunchKernelGGL((convert_matrix_kernel<bf16_t, true>), grid, blk, 0, ctx->stream, (const bf16_t*)s, dst, K, N, transposed, ldw, n_off);
        else hipLaunchKernelGGL((convert_matrix_kernel<bf16_t, false>), grid, blk, 0, ctx->stream, (const bf16_t*)s, dst, K, N, transposed, ldw, n_off);
      }
    };
    auto conv_vec = [&](const void* s, float* dst, size_t cnt) {
      dim3 grid((unsigned)((cnt + 255) / 256));
      if (T.dtype == BPD_F32) hipLaunchKernelGGL(convert_vector_kernel<float>, grid, blk, 0, ctx->stream, (const float*)s, dst, (long)cnt);
      else hipLaunchKernelGGL(convert_vector_kernel<bf16_t>, grid, blk, 0, ctx->stream, (const bf16_t*)s, dst, (long)cnt);
    };
    const size_t wsz = bf ? 2 : 4;
    switch (e.kind) {
      case VEC: conv_vec(src, (float*)e.dst, count); break;
      case MAT: conv_mat(src, e.dst, e.K, e.N, 0, e.ldw, e.n_off); break;
      case EMB:
        if (bf) conv_mat(src, e.dst, e.K, e.N, 1, e.ldw, 0);      // as the projection matrix W[d][V] = E^T
        else conv_vec(src, (float*)e.dst, count);                  // fp32 kernels read E[V][d] directly
        break;
      case MATK_CAT:
        for (int i = 0; i < (int)e.shape[0]; ++i)
          conv_mat((const char*)src + (size_t)i * e.K * e.N * esz, e.dst, e.K, e.N, 0, e.ldw, i * e.N);
        break;
      case MATK_SEP:
        for (int i = 0; i < (int)e.shape[0]; ++i)
          conv_mat((const char*)src + (size_t)i * e.K * e.N * esz, (char*)e.dst + (size_t)i * e.K * e.N * wsz, e.K, e.N, 0, e.ldw, 0);
        break;
    }
    LAUNCHCHK();
    HIPCHK(hipStreamSynchronize(ctx->stream));   // the staging area and the caller's buffer are free again
    e.loaded = true;
    ctx->fold_ready = false;
  }
  ctx->encoded = false;
  return BPD_OK;
}

int bpd_encode(bpd_ctx* ctx, const int32_t* src_ids, const int32_t* src_len, const int32_t* max_len, int B, int S) {
  if (!ctx || !src_ids || !src_len) return fail(ctx, BPD_E_ARG, "bpd_encode: null argument");
  const bpd_config& c = ctx->cfg;
  if (B < 1 || S < 1) return fail(ctx, BPD_E_ARG, "bpd_encode: B and S must be positive");
  if (B > c.max_batch || S > c.max_src_len) return fail(ctx, BPD_E_CAPACITY, "bpd_encode: batch or source length over the configured maximum");
  for (auto& kv : ctx->table)
    if (!kv.second.loaded) return fail(ctx, BPD_E_STATE, "bpd_encode: tensor not loaded: " + kv.first);
  // host-side validation when the caller's arrays are host memory
  if (is_host_ptr(src_len)) {
    for (int b = 0; b < B; ++b)
      if (src_len[b] < 1 || src_len[b] > S) return fail(ctx, BPD_E_ARG, "bpd_encode: src_len out of range");
  }
  if (is_host_ptr(src_ids)) {
    for (long i = 0; i < (long)B * S; ++i)
      if (src_ids[i] < 0 || src_ids[i] >= c.vocab) return fail(ctx, BPD_E_ARG, "bpd_encode: source id out of range");
  }
  if (max_len && is_host_ptr(max_len)) {
    for (int b = 0; b < B; ++b)
      if (max_len[b] < 1 || max_len[b] > c.max_out_len) return fail(ctx, BPD_E_ARG, "bpd_encode: max_len out of range");
  }
  Layout& L = ctx->lay;
  ctx->B = B; ctx->S = S; ctx->encoded = false; ctx->x_ready_k = 0;
  refresh_folded_weights(ctx);                    // (every tensor is loaded: checked above)
  HIPCHK(hipMemcpyAsync(L.src_ids, src_ids, (size_t)B * S * 4, hipMemcpyDefault, ctx->stream));
  HIPCHK(hipMemcpyAsync(L.src_len, src_len, (size_t)B * 4, hipMemcpyDefault, ctx->stream));
  if (max_len) HIPCHK(hipMemcpyAsync(L.max_len, max_len, (size_t)B * 4, hipMemcpyDefault, ctx->stream));
  else fill_i32(ctx, L.max_len, B, c.max_out_len);
  hipLaunchKernelGGL(sanitize_kernel, dim3((B * S + 255) / 256), dim3(256), 0, ctx->stream, L.src_len, L.max_len, L.src_ids, B, S,
                     c.max_out_len, c.vocab);
  int rc = encoder(ctx);
  if (rc) return rc;
  // empty hypotheses
  fill_i32(ctx, L.L, B, 0);
  fill_i32(ctx, L.j, B, 0);
  fill_i32(ctx, L.finished, B, 0);
  fill_i32(ctx, L.accepted, B, 0);
  fill_i32(ctx, L.out_ids, (long)B * c.max_out_len, c.pad_id);
  fill_i32(ctx, (int*)L.stats, 64, 0);
  fill_i32(ctx, L.P, (long)B * c.k_max, 0);
  fill_i32(ctx, L.A, (long)B * c.k_max * c.k_max, 0);
  // first invocation: position 0 only, all heads -> first proposals
  rc = forward(ctx, 1, c.k_max, 1, nullptr);
  if (rc) return rc;
  hipLaunchKernelGGL(prime_kernel, dim3(B), dim3(64), 0, ctx->stream, state_params(ctx), L.keys, B);
  LAUNCHCHK();
  ctx->steps = 0;
  ctx->encoded = true;
  return BPD_OK;
}

static int step_impl(bpd_ctx* ctx, int k, const int* imposed_dev, int imposed_stride, int imposed_step, int* accepted_dev) {
  Layout& L = ctx->lay;
  PhaseTimer whole(ctx, BPD_PHASE_STEP);
  ctx->cur_imposed = imposed_dev; ctx->cur_imposed_stride = imposed_stride; ctx->cur_imposed_step = imposed_step;
  int rc = forward(ctx, k, k, 0, nullptr);
  if (rc) return rc;
  {
    PhaseTimer t(ctx, BPD_PHASE_ACCEPT);
    StateP s = state_params(ctx);
    s.imposed = imposed_dev; s.imposed_stride = imposed_stride;
    const bpd_config& c = ctx->cfg;
    if (embed_in_accept(ctx)) {
      // the accept kernel also embeds the next block (same k assumed; checked by forward); its LayerNorm statistics go
      // where the first layer will look for them: the single-tile layout for at most 16 rows, per-tile rows otherwise
      const bool sp = stats_path(ctx, ctx->B * k);
      hipLaunchKernelGGL(accept_embed_kernel, dim3(ctx->B), dim3(1024), 0, ctx->stream, s, L.keys, k, ctx->B, imposed_step, accepted_dev,
                         c.d_model, (const bf16_t*)L.emb, c.vocab, (const float*)L.pos_tgt, sqrtf((float)c.d_model), L.x,
                         sp ? L.stats_ln : L.stats_big, sp ? 16 : ctx->B * k, sp ? (bf16_t*)nullptr : (bf16_t*)L.xn, (int)ctx->steps);
      ctx->x_ready_k = k;
    } else {
      hipLaunchKernelGGL(accept_kernel, dim3(ctx->B), dim3(64), 0, ctx->stream, s, L.keys, k, ctx->B, 1, imposed_step, accepted_dev, (int)ctx->steps);
      ctx->x_ready_k = 0;
    }
  }
  LAUNCHCHK();
  ctx->steps++;
  return BPD_OK;
}

int bpd_step(bpd_ctx* ctx, int k, const int32_t* imposed_accept, int32_t* accepted_len) {
  if (!ctx) return BPD_E_ARG;
  if (!ctx->encoded) return fail(ctx, BPD_E_STATE, "bpd_step: call bpd_encode first");
  if (k < 1 || k > ctx->cfg.k_max) return fail(ctx, BPD_E_ARG, "bpd_step: k outside 1..k_max");
  Layout& L = ctx->lay;
  // device pointers are used in place by the accept kernel; host arrays go through a copy
  const int* imp = nullptr;
  if (imposed_accept) {
    if (is_host_ptr_cached(ctx, imposed_accept)) {
      HIPCHK(hipMemcpyAsync(L.imposed1, imposed_accept, (size_t)ctx->B * 4, hipMemcpyHostToDevice, ctx->stream));
      imp = L.imposed1;
    } else {
      imp = imposed_accept;
    }
  }
  const bool out_host = accepted_len && is_host_ptr_cached(ctx, accepted_len);
  int rc = step_impl(ctx, k, imp, 0, 0, out_host ? nullptr : accepted_len);
  if (rc) return rc;
  if (out_host) HIPCHK(hipMemcpyAsync(accepted_len, L.accepted, (size_t)ctx->B * 4, hipMemcpyDeviceToHost, ctx->stream));
  return BPD_OK;
}

int bpd_step_static(bpd_ctx* ctx, int k, const int32_t* imposed_accept, int32_t* accepted_len) {
  if (!ctx) return BPD_E_ARG;
  if (!ctx->encoded) return fail(ctx, BPD_E_STATE, "bpd_step_static: call bpd_encode first");
  if (k < 1 || k > ctx->cfg.k_max) return fail(ctx, BPD_E_ARG, "bpd_step_static: k outside 1..k_max");
  Layout& L = ctx->lay;
  const bpd_config& c = ctx->cfg;
  char* sp = (char*)g_scratch_ptr[ctx->device];
  if (!sp) return fail(ctx, BPD_E_STATE, "bpd_step_static: no scratch address for this device");
  // what this step needs: its k x k keys per sequence, the head-1 / second-phase keys, the attention partials, and as
  // many K slices as bpd_step would use for the same block (so that both sum in the same order)
  const size_t M = (size_t)ctx->B * k, d = c.d_model;
  auto up = [](size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; };
  const size_t keys_b = up(M * k * 8), keys_h1_b = up(2 * M * 8);
  size_t attn_b = 0;                       // partial results of a split attention launch: splits x (head, sequence, row tile)
  for (int causal : {1, 0}) {
    const int ns = attention_nsplit(ctx, causal ? c.max_out_len + c.k_max + 1 : c.max_src_len, ctx->B, k, causal);
    const size_t wgs = (size_t)c.n_heads * ctx->B * ((k + 15) / 16);
    if (ns > 1) attn_b = std::max(attn_b, up(ns * wgs * 16 * (d / c.n_heads + 2) * 4));
  }
  size_t slices = 1;
  if (c.dtype == BPD_BF16 && M > 16)
    for (int K : {c.d_model, c.d_ff}) {
      const int ns = residual_k_slices(ctx, gp(nullptr, K, nullptr, c.d_model, (int)M, c.d_model, K));
      if ((size_t)ns > slices) slices = ns;
    }
  const size_t kpart_b = slices > 1 ? up(slices * M * d * 4) : 0;
  if (keys_b + keys_h1_b + attn_b + kpart_b > STATIC_SCRATCH_BYTES)
    return fail(ctx, BPD_E_CAPACITY, "bpd_step_static: this step needs " + std::to_string(keys_b + keys_h1_b + attn_b + kpart_b) +
                                     " bytes of scratch, the static array holds " + std::to_string(STATIC_SCRATCH_BYTES));
  const int* imp = nullptr;
  if (imposed_accept) {
    if (is_host_ptr_cached(ctx, imposed_accept)) {
      HIPCHK(hipMemcpyAsync(L.imposed1, imposed_accept, (size_t)ctx->B * 4, hipMemcpyHostToDevice, ctx->stream));
      imp = L.imposed1;
    } else {
      imp = imposed_accept;
    }
  }
  const bool out_host = accepted_len && is_host_ptr_cached(ctx, accepted_len);
  // the step's kernels take their scratch from the layout: point it at the static array for this call
  unsigned long long* const keys0 = L.keys; unsigned long long* const keys_h10 = L.keys_h1;
  float* const attn0 = L.attn_part; float* const kpart0 = L.kpart;
  L.keys = (unsigned long long*)sp;
  L.keys_h1 = (unsigned long long*)(sp + keys_b);
  L.attn_part = (float*)(sp + keys_b + keys_h1_b);
  L.kpart = (float*)(sp + keys_b + keys_h1_b + attn_b);
  // the array keeps the last call's contents and the keys are merged with atomic max: they start at zero
  // (a fill kernel, not a memset node: callers may be capturing the stream)
  fill_i32(ctx, (int*)L.keys, (long)(2 * M * k), 0);
  int rc = step_impl(ctx, k, imp, 0, 0, out_host ? nullptr : accepted_len);
  L.keys = keys0; L.keys_h1 = keys_h10; L.attn_part = attn0; L.kpart = kpart0;
  // (this step's accept kernel cleared the static keys, not the workspace's: the next step embeds its block and clears
  // its keys itself)
  ctx->x_ready_k = 0;
  if (rc) return rc;
  if (out_host) HIPCHK(hipMemcpyAsync(accepted_len, L.accepted, (size_t)ctx->B * 4, hipMemcpyDeviceToHost, ctx->stream));
  return BPD_OK;
}

int bpd_set_acceptance(bpd_ctx* ctx, int distance_eps, int min_block) {
  if (!ctx) return BPD_E_ARG;
  if (distance_eps < 0 || min_block < 1 || min_block > ctx->cfg.k_max) return fail(ctx, BPD_E_ARG, "bpd_set_acceptance: out of range");
  ctx->distance_eps = distance_eps; ctx->min_block = min_block;
  return BPD_OK;
}

int bpd_set_top_n(bpd_ctx* ctx, int n) {
  if (!ctx) return BPD_E_ARG;
  if (n < 1 || n > ctx->cfg.vocab) return fail(ctx, BPD_E_ARG, "bpd_set_top_n: n outside 1..vocab");
  ctx->top_n = n;
  return BPD_OK;
}

int bpd_set_two_phase(bpd_ctx* ctx, int on) {
  if (!ctx) return BPD_E_ARG;
  ctx->two_phase = on != 0;
  return BPD_OK;
}

int bpd_set_local_attention(bpd_ctx* ctx, int query_block, int memory_len) {
  if (!ctx) return BPD_E_ARG;
  if (query_block < 0 || memory_len < 0 || (query_block == 0 && memory_len != 0))
    return fail(ctx, BPD_E_ARG, "local attention: query_block >= 0, memory_len >= 0 (and 0 when query_block is 0)");
  ctx->local_q = query_block; ctx->local_m = memory_len;
  return BPD_OK;
}

int bpd_get_stats(bpd_ctx* ctx, bpd_stats* st) {
  if (!ctx || !st) return BPD_E_ARG;
  long long raw[32];
  HIPCHK(hipMemcpyAsync(raw, ctx->lay.stats, sizeof(raw), hipMemcpyDeviceToHost, ctx->stream));
  HIPCHK(hipStreamSynchronize(ctx->stream));
  st->steps = raw[20]; st->invocations = ctx->encoded ? raw[20] + 1 : 0;
  st->seq_steps = raw[0]; st->accepted_total = raw[1]; st->finished = (int32_t)raw[2];
  for (int i = 0; i < 17; ++i) st->hist[i] = raw[3 + i];
  return BPD_OK;
}

int bpd_get_output(bpd_ctx* ctx, int32_t* out_ids, int32_t* out_len) {
  if (!ctx) return BPD_E_ARG;
  if (!ctx->encoded) return fail(ctx, BPD_E_STATE, "bpd_get_output: nothing decoded");
  Layout& L = ctx->lay;
  if (out_ids) HIPCHK(hipMemcpyAsync(out_ids, L.out_ids, (size_t)ctx->B * ctx->cfg.max_out_len * 4, hipMemcpyDefault, ctx->stream));
  if (out_len) HIPCHK(hipMemcpyAsync(out_len, L.j, (size_t)ctx->B * 4, hipMemcpyDefault, ctx->stream));
  HIPCHK(hipStreamSynchronize(ctx->stream));
  return stack_check(ctx);
}

int bpd_decode(bpd_ctx* ctx, int k, const int32_t* schedule, int max_steps, int32_t* out_ids, int32_t* out_len, bpd_stats* stats) {
  if (!ctx) return BPD_E_ARG;
  if (!ctx->encoded) return fail(ctx, BPD_E_STATE, "bpd_decode: call bpd_encode first");
  if (k < 1 || k > ctx->cfg.k_max || max_steps < 0) return fail(ctx, BPD_E_ARG, "bpd_decode: bad k or max_steps");
  Layout& L = ctx->lay;
  const int B = ctx->B;
  const int* imp = nullptr;
  if (schedule) {
    // a live sequence takes at least one token per step, so max_out_len rows always suffice
    const int rows = max_steps < ctx->cfg.max_out_len ? max_steps : ctx->cfg.max_out_len;
    if (rows > 0) HIPCHK(hipMemcpyAsync(L.sched, schedule, (size_t)rows * B * 4, hipMemcpyDefault, ctx->stream));
    if (max_steps > rows) max_steps = rows;
    imp = L.sched;
  }
  for (int s = 0; s < max_steps; ++s) {
    int rc = step_impl(ctx, k, imp, B, s, nullptr);
    if (rc) return rc;
    if ((s & 3) == 3 || s + 1 == max_steps) {
      HIPCHK(hipMemcpyAsync(ctx->pinned, (int*)(L.stats + 2), 4, hipMemcpyDeviceToHost, ctx->stream));
      HIPCHK(hipStreamSynchronize(ctx->stream));
      if (ctx->pinned[0] >= B) break;
    }
  }
  int rc = bpd_get_output(ctx, out_ids, out_len);
  if (rc) return rc;
  if (stats) return bpd_get_stats(ctx, stats);
  return BPD_OK;
}

int bpd_get_state(bpd_ctx* ctx, int32_t* P, int32_t* A, int32_t* j, int32_t* finished) {
  if (!ctx) return BPD_E_ARG;
  if (!ctx->encoded) return fail(ctx, BPD_E_STATE, "bpd_get_state: call bpd_encode first");
  Layout& L = ctx->lay;
  const size_t B = ctx->B, k = ctx->cfg.k_max;
  if (P) HIPCHK(hipMemcpyAsync(P, L.P, B * k * 4, hipMemcpyDefault, ctx->stream));
  if (A) HIPCHK(hipMemcpyAsync(A, L.A, B * k * k * 4, hipMemcpyDefault, ctx->stream));
  if (j) HIPCHK(hipMemcpyAsync(j, L.j, B * 4, hipMemcpyDefault, ctx->stream));
  if (finished) HIPCHK(hipMemcpyAsync(finished, L.finished, B * 4, hipMemcpyDefault, ctx->stream));
  HIPCHK(hipStreamSynchronize(ctx->stream));
  return stack_check(ctx);
}

int bpd_set_proposals(bpd_ctx* ctx, const int32_t* P) {
  if (!ctx || !P) return fail(ctx, BPD_E_ARG, "bpd_set_proposals: null argument");
  if (!ctx->encoded) return fail(ctx, BPD_E_STATE, "bpd_set_proposals: call bpd_encode first");
  const size_t n = (size_t)ctx->B * ctx->cfg.k_max;
  if (is_host_ptr(P)) {
    for (size_t i = 0; i < n; ++i)
      if (P[i] < 0 || P[i] >= ctx->cfg.vocab) return fail(ctx, BPD_E_ARG, "bpd_set_proposals: token id out of range");
  }
  HIPCHK(hipMemcpyAsync(ctx->lay.P, P, n * 4, hipMemcpyDefault, ctx->stream));
  ctx->x_ready_k = 0;              // a block embedded ahead of time used the old proposals
  return BPD_OK;
}

int bpd_debug_step_logits(bpd_ctx* ctx, int k, float* logits) {
  if (!ctx || !logits) return fail(ctx, BPD_E_ARG, "bpd_debug_step_logits: null argument");
  if (!ctx->encoded) return fail(ctx, BPD_E_STATE, "bpd_debug_step_logits: call bpd_encode first");
  if (k < 1 || k > ctx->cfg.k_max) return fail(ctx, BPD_E_ARG, "bpd_debug_step_logits: k outside 1..k_max");
  int rc = forward(ctx, k, k, 0, logits);
  if (rc) return rc;
  hipLaunchKernelGGL(accept_kernel, dim3(ctx->B), dim3(64), 0, ctx->stream, state_params(ctx), ctx->lay.keys, k, ctx->B, 0, 0, nullptr, 0);
  LAUNCHCHK();
  return BPD_OK;
}

int bpd_profile_enable(bpd_ctx* ctx, int phase) {
  if (!ctx || phase < 0 || phase > BPD_PHASE_EMPTY) return BPD_E_ARG;
  (void)hipStreamSynchronize(ctx->stream);
  ctx->prof_phase = phase; ctx->prof_used = 0; ctx->prof_launches = 0;
  return BPD_OK;
}

int bpd_profile_read(bpd_ctx* ctx, double* total_ms, int64_t* launches) {
  if (!ctx || !total_ms || !launches) return BPD_E_ARG;
  return bpd_profile_samples(ctx, nullptr, 0, total_ms, launches);
}

int bpd_profile_samples(bpd_ctx* ctx, float* ms_out, int64_t capacity, double* total_ms, int64_t* launches) {
  if (!ctx || !total_ms || !launches || capacity < 0 || (capacity > 0 && !ms_out)) return BPD_E_ARG;
  HIPCHK(hipStreamSynchronize(ctx->stream));
  double tot = 0;
  int64_t n = 0;
  for (size_t i = 0; i + 1 < ctx->prof_used; i += 2, ++n) {
    float ms = 0.f;
    HIPCHK(hipEventElapsedTime(&ms, ctx->prof_ev[i], ctx->prof_ev[i + 1]));
    tot += ms;
    if (n < capacity) ms_out[n] = ms;
  }
  *total_ms = tot; *launches = ctx->prof_launches;
  ctx->prof_used = 0; ctx->prof_launches = 0;
  return BPD_OK;
}

// ------------------------------------------------------------------------------- machine peaks

int bpd_measure_hbm_read(void* buf_dev, size_t bytes, void* hip_stream, int iters, double* gbps) {
  if (!buf_dev || !gbps || iters < 1 || bytes < (1u << 20) || bytes % 4096 != 0) return BPD_E_ARG;
  hipStream_t s = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return BPD_E_HIP;
  const long n16 = (long)(bytes / 16);
  double best = 0;
  for (int rep = 0; rep < 3; ++rep) {
    (void)hipEventRecord(e0, s);
    for (int i = 0; i < iters; ++i)
      hipLaunchKernelGGL(peak_read_kernel, dim3(2048), dim3(256), 0, s, (const uint4*)buf_dev, n16, (unsigned*)buf_dev);
    (void)hipEventRecord(e1, s);
    if (hipStreamSynchronize(s) != hipSuccess) return BPD_E_HIP;
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    const double r = (double)bytes * iters / (ms * 1e6);
    if (rep > 0 && r > best) best = r;
  }
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  *gbps = best;
  return BPD_OK;
}

int bpd_measure_mfma_bf16(void* scratch_dev, void* hip_stream, int iters, double* tflops) {
  if (!scratch_dev || !tflops || iters < 1) return BPD_E_ARG;
  hipStream_t s = (hipStream_t)hip_stream;
  hipEvent_t e0, e1;
  if (hipEventCreate(&e0) != hipSuccess || hipEventCreate(&e1) != hipSuccess) return BPD_E_HIP;
  int dev = 0, cus = 0;
  (void)hipGetDevice(&dev);
  (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  const int wgs = 2 * cus;                     // two 4-wave workgroups per CU: two waves per SIMD
  double best = 0;
  for (int rep = 0; rep < 3; ++rep) {
    (void)hipEventRecord(e0, s);
    hipLaunchKernelGGL(peak_mfma_kernel, dim3(wgs), dim3(256), 0, s, (float*)scratch_dev, iters, 1u + rep);
    (void)hipEventRecord(e1, s);
    if (hipStreamSynchronize(s) != hipSuccess) return BPD_E_HIP;
    float ms = 0.f;
    (void)hipEventElapsedTime(&ms, e0, e1);
    const double r = (double)wgs * 4 * iters * 16 * 16384.0 / (ms * 1e9);
    if (rep > 0 && r > best) best = r;
  }
  (void)hipEventDestroy(e0); (void)hipEventDestroy(e1);
  *tflops = best;
  return BPD_OK;
}

}  // extern "C"
