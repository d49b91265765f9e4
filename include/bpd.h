/*
 * libbpd — blockwise parallel decoding (Stern, Shazeer, Uszkoreit, NeurIPS 2018) on one
 * MI355X (gfx950).  C ABI: plain pointers and sizes, no C++ or torch types.
 *
 * The library implements the decoding loop of the paper's Sections 3 and 4 for the combined
 * scoring-and-proposal model of Section 6:
 *
 *   given a source x, keep a hypothesis y-hat of length j and k proposals P_1..P_k for the
 *   next k tokens; one model invocation scores the k proposed positions against the cached
 *   prefix and yields, at every block row i' and for every head i, the argmax
 *   A[i'][i] of p_i(y_{j+i'+i} | y-hat_{<=j}, P_1..P_i', x); the longest prefix of P that the
 *   base model p_1 would have produced greedily is appended (k-hat tokens, 1 <= k-hat <= k)
 *   and row k-hat of A becomes the next block of proposals.
 *
 * All device work is enqueued on the HIP stream given at creation; unless stated otherwise a
 * call does not synchronise.  Every function returns 0 (BPD_OK) or a negative error code and
 * never throws or aborts; bpd_last_error() gives a message.  On an argument error the decode
 * state is left unchanged.
 *
 * Calls on one context must not overlap (one thread at a time, or external locking), and all
 * contexts of a process must live on one device: kernel attributes are set once per process.
 *
 * Pointer arguments marked [host|device] may be either (they are copied with
 * hipMemcpyDefault); arguments marked [device] are dereferenced by kernels.
 */
#ifndef BPD_H
#define BPD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define BPD_OK           0
#define BPD_E_ARG       (-1)  /* null pointer, size out of range, k > k_max, ...            */
#define BPD_E_STATE     (-2)  /* call out of order: step before encode, encode before load  */
#define BPD_E_CAPACITY  (-3)  /* workspace too small, batch / source length over the limits */
#define BPD_E_WEIGHTS   (-4)  /* unknown tensor name, wrong shape, tensors missing           */
#define BPD_E_HIP       (-5)  /* a HIP runtime call or kernel launch failed                  */

#define BPD_F32  0
#define BPD_BF16 1

typedef struct bpd_ctx bpd_ctx;   /* opaque; owns small host structs only */

/* Model and capacity description.  k_max counts all heads p_1..p_k (Section 3: p_1 is the
 * base model, p_2..p_k the proposal models; Section 6: p_1 passes through a head as well).
 *
 * Accepted shapes (anything else makes bpd_workspace_bytes return 0 and bpd_create BPD_E_ARG):
 *   n_enc_layers, n_dec_layers, n_heads, max_batch, max_src_len, max_out_len >= 1;
 *   1 <= k_max <= 16;
 *   d_model a multiple of 32 and of n_heads, 32 <= d_model <= 2048;
 *   head width d_model / n_heads = 16 or 64 (BPD_BF16), 16 only (BPD_F32: meant for small models);
 *   d_ff a multiple of 32;  vocab a multiple of 16, >= 16;
 *   dtype BPD_F32 or BPD_BF16;  eos_id < vocab;  ln_eps > 0. */
typedef struct {
  int32_t n_enc_layers, n_dec_layers;
  int32_t d_model, n_heads, d_ff, vocab;
  int32_t k_max;                      /* number of heads = largest block size, <= 16        */
  int32_t max_batch, max_src_len, max_out_len;
  int32_t dtype;                      /* BPD_F32: fp32 everywhere.  BPD_BF16: bf16 weights,
                                         bf16 K/V caches and GEMM inputs, fp32 accumulation,
                                         fp32 residual stream / LayerNorm / softmax          */
  int32_t eos_id;                     /* < 0: fixed-length decoding (Section 2, images)      */
  int32_t pad_id;                     /* fills out_ids beyond out_len                        */
  float   ln_eps;
} bpd_config;

/* One named weight tensor handed to bpd_load_weights.  Row-major, shape[0..ndim).  Matrices
 * are input-major (y = x W, W[in][out]).  Names (l = layer index):
 *   emb [V,d]   pos_src [max_src_len,d]   pos_tgt [max_out_len+k_max+1,d]
 *   enc.l.ln1.g/.b [d]  enc.l.self.wq/.wk/.wv/.wo [d,d]  enc.l.ln2.g/.b  enc.l.ffn.w1 [d,F] .b1 [F] .w2 [F,d] .b2 [d]
 *   enc.lnf.g/.b
 *   dec.l.ln1.g/.b  dec.l.self.wq/.wk/.wv/.wo  dec.l.ln2.g/.b  dec.l.cross.wq/.wk/.wv/.wo
 *   dec.l.ln3.g/.b  dec.l.ffn.w1/.b1/.w2/.b2      dec.lnf.g/.b
 *   head.w1 [k_max,d,F]  head.b1 [k_max,F]  head.w2 [k_max,F,d]  head.b2 [k_max,d]   (Section 6) */
typedef struct {
  const char* name;
  const void* data;        /* [host|device], see on_device                                  */
  int32_t dtype;           /* BPD_F32 (float) or BPD_BF16 (uint16 bit patterns)             */
  int32_t ndim;
  int64_t shape[4];
  int32_t on_device;       /* 0: host memory, 1: device memory                              */
} bpd_tensor;

/* Counters since the last bpd_encode (they run on over several bpd_step / bpd_decode calls).
 * mean accepted block size (Section 7.1) =
 * accepted_total / (steps summed over live sequences) = accepted_total / seq_steps.        */
typedef struct {
  int64_t steps;           /* steps in which at least one sequence was still decoding       */
  int64_t invocations;     /* model invocations = steps + 1 (Section 4)                     */
  int64_t seq_steps;       /* sum over steps of sequences still decoding                    */
  int64_t accepted_total;  /* sum of k-hat over sequences and steps                         */
  int64_t hist[17];        /* hist[a] = number of (sequence, step) pairs with k-hat = a     */
  int32_t finished;        /* sequences that have ended                                     */
} bpd_stats;

/* Bytes of device workspace bpd_create needs for this configuration (weights in kernel
 * layout -- with max_batch * k_max > 128 in bf16 mode also copies of three decoder matrices
 * per layer with their LayerNorm folded in --, K/V caches, activations, decode state, a
 * staging area for host weights).
 * Returns 0 if the configuration is invalid. */
size_t bpd_workspace_bytes(const bpd_config* cfg);

/* Create a context on the current device.  workspace [device] is caller-owned, 256-byte
 * aligned, at least bpd_workspace_bytes(cfg) bytes, and must outlive the context; the
 * library allocates no device memory itself.  hip_stream is a hipStream_t (NULL = the
 * default stream).  Errors: BPD_E_ARG, BPD_E_CAPACITY. */
int bpd_create(const bpd_config* cfg, void* workspace, size_t workspace_bytes,
               void* hip_stream, bpd_ctx** out);
int bpd_destroy(bpd_ctx* ctx);

/* The parameters of the combined model of Section 6 (Figure 3): the encoder-decoder Transformer
 * that is p_1's body, and on top of its decoder output one inserted feed-forward layer per head
 * with a residual connection, all heads sharing the vocabulary projection (the tensor names are
 * listed at bpd_tensor).
 * Copy n named tensors into the workspace, converting to the kernel layout (bf16 MFMA tiles
 * in BPD_BF16 mode).  The caller's buffers are not referenced after the call returns
 * (the call synchronises the stream).  May be called several times; every tensor must have
 * been loaded before bpd_encode, and a call made after bpd_encode ends the decode in progress
 * (bpd_step then returns BPD_E_STATE until the next bpd_encode).  All n tensors are validated
 * (name, shape, dtype, staging capacity) before the first is copied: a call that fails leaves
 * the loaded set as it was.
 * Errors: BPD_E_WEIGHTS (unknown name / shape / dtype), BPD_E_CAPACITY, BPD_E_ARG. */
int bpd_load_weights(bpd_ctx* ctx, const bpd_tensor* tensors, int n);

/* Condition on a batch of sources (Section 2: the input x) and start decoding:
 * runs the encoder, fills the cross-attention K/V, resets the hypotheses (j = 0), and makes
 * the first model invocation on the empty prefix, whose k_max argmaxes become the first
 * proposals (the "+1" invocation of Section 4).
 *   src_ids [host|device]  int32 [B, S] row-major, rows padded beyond src_len[b]
 *   src_len [host|device]  int32 [B], 1 <= src_len[b] <= S
 *   max_len [host|device]  int32 [B] output budget per sequence (1..max_out_len), or NULL
 * Errors: BPD_E_STATE (weights missing), BPD_E_CAPACITY (B, S over the limits), BPD_E_ARG. */
int bpd_encode(bpd_ctx* ctx, const int32_t* src_ids, const int32_t* src_len,
               const int32_t* max_len, int B, int S);

/* One combined verify + predict step with block size k (Sections 3 and 4), 1 <= k <= k_max,
 * the same k on every step of a decode.
 *   imposed_accept [host|device] int32 [B] or NULL.  NULL: exact-match verification
 *       (k-hat = longest prefix of P equal to p_1's argmaxes).  Otherwise the verify outcome
 *       is replaced by imposed_accept[b] (clamped to 1..k); the accepted tokens are still
 *       P_1..P_k-hat and the next proposals still row k-hat of A.  Not in the paper: it lets
 *       untrained heads exercise every accepted length.
 *   accepted_len [host|device] int32 [B] or NULL: k-hat per sequence after the cut at the
 *       first EOS (inclusive, cf. Section 7.4) and at max_len; 0 for sequences that had
 *       already ended.  With a pageable host pointer the call waits for the copy.
 * Errors: BPD_E_STATE (no bpd_encode yet), BPD_E_ARG. */
int bpd_step(bpd_ctx* ctx, int k, const int32_t* imposed_accept, int32_t* accepted_len);

/* bpd_step for callers that cannot allocate device memory and cannot spare workspace for a step's scratch: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same results (the
 * same kernels in the same order) and the same state transition as bpd_step; the scratch of the step (arg-max keys
 * merged by atomic max, split-KV attention partials, split-K slices) lives in an 8 MiB array inside the library's
 * device image instead of the workspace.  The call allocates nothing (no hipMalloc / hipFree, no allocating library
 * routine) and clears what must start at zero with a fill kernel.  Every context on a GPU shares that GPU's array and
 * it keeps the last call's contents: calls that overlap on one GPU (other streams, other threads) race.
 * Errors: as bpd_step, and BPD_E_CAPACITY when the step's scratch exceeds the array (8 k^2 B bytes of keys, up to
 * 2.2 MB of attention partials once a cache is long enough to be split, the K slices of blocks of more than 16 rows;
 * Transformer-big at batch 32, k = 10 needs 5.3 MB), with the byte counts in bpd_last_error(). */
int bpd_step_static(bpd_ctx* ctx, int k, const int32_t* imposed_accept, int32_t* accepted_len);

/* Relaxed verification (Section 5), applies to later bpd_step / bpd_decode calls with
 * imposed_accept == NULL:  a proposal is accepted if |P - argmax p_1| <= distance_eps
 * (Section 5.2; 0 = exact match) and at least min_block tokens are taken (Section 5.3;
 * 1 = no minimum).  Errors: BPD_E_ARG. */
int bpd_set_acceptance(bpd_ctx* ctx, int distance_eps, int min_block);

/* Top-n verification (Section 5.1), applies to later bpd_step / bpd_decode calls with
 * imposed_accept == NULL: a proposal is also accepted if it is among the n highest-scoring
 * tokens of p_1 at its block row (ties go to the lower token id, as in the arg-max).  n = 1
 * switches the criterion off (exact match, or whatever bpd_set_acceptance selected; the two
 * criteria are OR-ed).  With n > 1 every step scores p_1 of the k block rows a second time with
 * the logits kept in the workspace ([B*k, vocab] fp32), so a step costs one more pass over the
 * embedding matrix.  Errors: BPD_E_ARG (n outside 1..vocab). */
int bpd_set_top_n(bpd_ctx* ctx, int n);

/* Two-phase scoring (a variant of the combined model of Section 4 that yields the same tokens):
 * with on != 0 a step scores p_1 at the k block rows first, verifies, and then evaluates the
 * heads 2..k only at block row k-hat, the one row whose proposals the next step uses: 2k - 1
 * vocabulary-projection rows per sequence instead of k^2, at the price of a second, dependent
 * pass over the head and embedding weights.  Pays off when the step is compute bound (large
 * batch); applies to bf16 contexts with more than 16 block rows per step, otherwise ignored.
 * The table returned by bpd_get_state then holds column 1 of every row and row k-hat only
 * (other entries -1).  Default off.  Errors: BPD_E_ARG (null ctx). */
int bpd_set_two_phase(bpd_ctx* ctx, int on);

/* 1D local self-attention in the decoder (the attention layer of the image model of Section 7.2;
 * the paper names it without giving lengths).  Target positions are cut into consecutive query
 * blocks of query_block positions; the row at position t attends to
 *     floor(t / query_block) * query_block - memory_len  ..  t
 * (clipped at 0): its own block, causally, and the memory_len positions before the block.
 * query_block = 0 (then memory_len must be 0) restores full causal attention, the default.
 * The cache keeps every row either way, so the setting may change between steps; it applies to
 * later bpd_encode / bpd_step / bpd_decode / bpd_debug_step_logits calls.  Encoder and
 * cross-attention are not affected.  Errors: BPD_E_ARG (null ctx, negative lengths). */
int bpd_set_local_attention(bpd_ctx* ctx, int query_block, int memory_len);

/* The decoding loop of Section 3 with the merged verify / predict invocation of Section 4:
 * repeat bpd_step until every sequence has ended or max_steps steps were made; synchronises.
 * A sequence ends as greedy decoding does (Section 2): when the end-of-sequence token has been
 * accepted, or at its length budget max_len (the only rule when eos_id < 0: a fixed number of
 * tokens, as for the images of Section 7.2).
 *   schedule [host|device] int32 [max_steps, B] imposed accepted lengths, or NULL
 *   out_ids  [host|device] int32 [B, max_out_len], pad_id beyond out_len[b]
 *   out_len  [host|device] int32 [B]
 *   stats    host pointer or NULL
 * Errors: as bpd_step. */
int bpd_decode(bpd_ctx* ctx, int k, const int32_t* schedule, int max_steps,
               int32_t* out_ids, int32_t* out_len, bpd_stats* stats);

/* Copy out the decode state (synchronises).  Any pointer may be NULL.  [host|device].
 *   P [B,k_max] current proposals; A [B,k_max,k_max] argmax table of the last invocation
 *   (A[b][i'][i] = head i+1 at block row i'+1); j [B] accepted lengths; finished [B] flags. */
int bpd_get_state(bpd_ctx* ctx, int32_t* P, int32_t* A, int32_t* j, int32_t* finished);
int bpd_get_output(bpd_ctx* ctx, int32_t* out_ids, int32_t* out_len);
int bpd_get_stats(bpd_ctx* ctx, bpd_stats* stats);

/* Overwrite the current proposals P [host|device] int32 [B, k_max] (teacher forcing: lets a
 * test drive the cache along a given token sequence). */
int bpd_set_proposals(bpd_ctx* ctx, const int32_t* P);

/* Run the model invocation of the next step with block size k WITHOUT verifying or
 * committing, and write all logits: logits [device] float [B, k, k, vocab],
 * logits[b][i'][i][v] = score of head i+1 at block row i'+1.  The argmax table A is
 * refreshed as by bpd_step; j, P and the caches' committed part are unchanged. */
int bpd_debug_step_logits(bpd_ctx* ctx, int k, float* logits);

/* Timing hook for benchmarks: when enabled, bpd_step brackets the kernels of one phase
 * (BPD_PHASE_*) with HIP events on the context's stream; bpd_profile_read synchronises and
 * returns the accumulated milliseconds and the number of launches since it was enabled. */
#define BPD_PHASE_NONE         0
#define BPD_PHASE_LAYERS       1   /* decoder layers (embedding .. final LayerNorm), many kernels */
#define BPD_PHASE_HEAD_HIDDEN  2   /* heads, hidden layers: one GEMM kernel                       */
#define BPD_PHASE_HEAD_OUT     3   /* heads, k output layers + residual: one grouped GEMM kernel  */
#define BPD_PHASE_VOCAB        4   /* vocabulary projection + argmax: one kernel                  */
#define BPD_PHASE_ACCEPT       5   /* verify / accept / commit                                    */
#define BPD_PHASE_STEP         6   /* the whole step                                              */
#define BPD_PHASE_EMPTY        7   /* nothing: two events back to back, what the bracketing itself costs */
int bpd_profile_enable(bpd_ctx* ctx, int phase);
int bpd_profile_read(bpd_ctx* ctx, double* total_ms, int64_t* launches);
/* As bpd_profile_read, and additionally copies the milliseconds of the first `capacity` launches,
 * in launch order, to ms_out [host] (for latency percentiles).  Errors: BPD_E_ARG, BPD_E_HIP. */
int bpd_profile_samples(bpd_ctx* ctx, float* ms_out, int64_t capacity, double* total_ms, int64_t* launches);

/* Measured peaks of the machine, for roofline denominators next to the published ones (not part
 * of the method; no context needed).  Both launch on hip_stream, synchronise it and allocate
 * nothing.
 *   bpd_measure_hbm_read:  `iters` streaming-read passes over buf_dev [device, bytes, a multiple
 *       of 4096 and >= 1 MiB, contents irrelevant, not modified]; *gbps = best of two timed
 *       repetitions.  Use a buffer larger than the 256 MB last-level cache for an HBM figure.
 *   bpd_measure_mfma_bf16: back-to-back v_mfma_f32_16x16x32_bf16 with pseudo-random operands, two
 *       waves per SIMD, `iters` x 16 per wave; scratch_dev [device, >= 4 bytes]; *tflops = best of
 *       two timed repetitions.
 * Errors: BPD_E_ARG, BPD_E_HIP. */
int bpd_measure_hbm_read(void* buf_dev, size_t bytes, void* hip_stream, int iters, double* gbps);
int bpd_measure_mfma_bf16(void* scratch_dev, void* hip_stream, int iters, double* tflops);

const char* bpd_last_error(const bpd_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* BPD_H */
