/*
 * first.h -- C ABI of the MI355X (gfx950) implementation of FiRST's inference hot path:
 * router-gated prefill and autoregressive decode of a Llama-style decoder.
 *
 * Method (paper sections in parentheses):
 *   - every decoder layer i has a router R_i: a bias-free linear map D->1 applied to each
 *     token of the stream entering the layer, a sigmoid per token and a mean over the
 *     sequence, giving rho_i in [0,1] per sequence (Section 4.1);
 *   - the layer is kept iff rho_i >= 0.5; a skipped layer passes the hidden state of its
 *     nearest kept ancestor through unchanged (Section 3, Eq. 2 and its rounded form);
 *   - prefill never skips, so the first generated token is the full model's, and the
 *     decisions taken in prefill are cached and followed by every decode token, so a kept
 *     layer always holds KV for all earlier positions and a skipped layer needs none
 *     (Section 4.3, items 1 and 2).
 *
 * Conventions
 *   - "DEV" pointers are device (HBM) addresses, "HOST" pointers are host addresses.
 *   - All matrices are row-major [out_features, in_features]; bf16 is the raw upper half
 *     of an IEEE fp32; the residual stream, router, logits and all accumulation are fp32.
 *   - The caller owns weights, token buffers and every output buffer; weights are borrowed
 *     for the life of the context.  The library owns the paged KV cache, page tables, the
 *     mask / kept-index store, workspaces and cached hipGraphs.
 *   - All device work is enqueued on the hipStream_t given at creation and is asynchronous
 *     with respect to the host unless stated.  One context per stream; not re-entrant.
 *   - Every entry point returns FIRST_OK (0) or a negative error code and never throws or
 *     aborts; on an argument/state/capacity error nothing has been enqueued and no output
 *     is written.  first_last_error() gives the text of the last failure.
 */
#ifndef FIRST_H_
#define FIRST_H_

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FIRST_OK            0
#define FIRST_ERR_ARG      -1   /* null / out-of-range / misaligned argument               */
#define FIRST_ERR_STATE    -2   /* call not legal in the current state of the sequence(s)  */
#define FIRST_ERR_CAPACITY -3   /* batch, sequence length or KV pages exceed the context   */
#define FIRST_ERR_HIP      -4   /* a HIP runtime call failed (text in first_last_error)    */

#define FIRST_DTYPE_FP32 0
#define FIRST_DTYPE_BF16 1

/* options for first_set_option */
#define FIRST_OPT_USE_GRAPH     1  /* 1 (default): a decode step is a cached hipGraph (one per set of masks on the per-op and batched
                                      paths; a single one on the persistent path, whose kernel reads the kept layers from
                                      the device); 0: eager launches */
#define FIRST_OPT_ATTN_SPLITS   2  /* KV splits per (sequence, KV head) in decode attention; 0 = auto   */
#define FIRST_OPT_DECODE_PATH   3  /* -1 (default): persistent whole-step kernel when the model fits it
                                      (bf16, widths multiples of 256, one live sequence), else per-op
                                      kernels; 0: always per-op kernels; 1: persistent kernel or error.
                                      When device memory allows, first_create gives the persistent kernel a copy of every
                                      layer's down-projection matrix with permuted columns (as much memory again as those
                                      matrices); the caller's matrices must then not change after first_create. */

#define FIRST_OPT_STEP_TIMING   4  /* 1: the persistent kernel records per-phase timestamps (first_step_timing) */
#define FIRST_OPT_BATCH_TILED   9  /* batched decode: 1 (default when max_batch > 1 and device memory allows) = the mat-vecs
                                      read copies of the matrices in MFMA tile order, made at first_create (as much memory
                                      again as the weights; the caller's matrices must not change afterwards); 0 = they
                                      read the caller's row-major matrices */
#define FIRST_OPT_PREFILL_ATTN  7  /* prompt attention.  1 (default): tiled kernel on the matrix cores when the cache is bf16
                                      and head_dim is 64 or 128, else the plain kernel; 0: always the plain fp32 kernel */
#define FIRST_OPT_STEP_POLL_LIMIT 10 /* test tap: value >= 0 = the number of unsuccessful polls after which a wait between workgroups of
                                      the persistent kernel gives up (default, or -1: 2^21, seconds).  With 0 the next decode step
                                      gives up at its first exchange: every wave leaves at its next wait, nothing hangs, and the next
                                      call that synchronises (first_sync, first_seq_len, ...) returns FIRST_ERR_HIP, clears the limit
                                      and resets the exchange state; the live sequences must be prefilled again.  Synchronises. */
#define FIRST_OPT_BATCH_PATH    6  /* decode with several live sequences.  -1 (default): per layer, the sequences that
                                      keep it share one pass over its weights (bf16 models, widths multiples of 8),
                                      else one pass per sequence; 0: always one pass per sequence; 1: shared pass or error */

typedef struct first_ctx first_ctx;

/* Geometry of the decoder.  POD, filled by the caller. */
typedef struct first_model_desc {
  int32_t n_layers;       /* L (m in the paper)                                            */
  int32_t d_model;        /* D, multiple of 8                                              */
  int32_t n_q_heads;      /* Hq, multiple of n_kv_heads                                    */
  int32_t n_kv_heads;     /* Hkv                                                           */
  int32_t head_dim;       /* 64 or 128                                                     */
  int32_t d_ffn;          /* F, multiple of 8                                              */
  int32_t vocab;          /* V                                                             */
  int32_t dtype;          /* FIRST_DTYPE_*: storage type of the weights and of the KV cache */
  float   rope_base;      /* rotate-half RoPE, theta_d = base^(-2d/head_dim)               */
  float   rms_eps;        /* RMSNorm epsilon                                               */
  int32_t kv_page_tokens; /* tokens per KV page (16)                                       */
  int32_t max_batch;      /* sequences the context can hold at once                        */
  int32_t max_seq_len;    /* prompt + generated tokens per sequence                        */
  int32_t kv_layer_slots; /* 0 (or >= n_layers): KV pages for every layer.  1..n_layers-1:
                           * skip-aware KV elision, see first_create                         */
} first_model_desc;

/* Weights.  The struct and the per-layer pointer arrays are HOST memory (copied at create);
 * every pointer inside is DEV memory of the model's dtype except where marked fp32. */
typedef struct first_weights {
  const void *embed;               /* [V, D]                                               */
  const void *lm_head;             /* [V, D], untied                                       */
  const float *final_norm;         /* [D] fp32 gains                                       */
  const float *const *attn_norm;   /* [L] -> [D] fp32                                      */
  const void *const *wq;           /* [L] -> [Hq*hd, D]                                    */
  const void *const *wk;           /* [L] -> [Hkv*hd, D]                                   */
  const void *const *wv;           /* [L] -> [Hkv*hd, D]                                   */
  const void *const *wo;           /* [L] -> [D, Hq*hd]                                    */
  const float *const *mlp_norm;    /* [L] -> [D] fp32                                      */
  const void *const *w_gate;       /* [L] -> [F, D]                                        */
  const void *const *w_up;         /* [L] -> [F, D]                                        */
  const void *const *w_down;       /* [L] -> [D, F]                                        */
  const float *router;             /* [L, D] fp32, no bias (Section 4.1)                   */
} first_weights;

/* Creates a context: validates the geometry, allocates the KV page pool
 * (max_batch * ceil(max_seq_len / kv_page_tokens) pages per layer), page tables and
 * workspaces.  hip_stream is a hipStream_t; NULL makes the context create a private stream
 * that keeps the null stream's implicit ordering (graphs cannot be captured on the null
 * stream itself).
 *
 * Skip-aware KV elision (kv_layer_slots in 1..n_layers-1).  Router i reads the input of
 * layer i (Section 4.1), so its decision is known before the layer stores anything, and decode
 * never reads the KV of a layer it skips (Section 4.3 item 2).  The pool then holds
 * kv_layer_slots layer slices plus one scratch slice instead of n_layers slices: during
 * first_prefill_route a layer receives a slice when the first sequence's router keeps it, and
 * the prompt pass of a layer no sequence keeps (prefill never skips) puts its K/V in the
 * scratch slice, overwritten by the next such layer.  Slices are per layer, shared by the live
 * sequences: the memory used is (number of layers kept by at least one sequence + 1) slices.
 * If the routers keep more layers than there are slots first_prefill_route returns
 * FIRST_ERR_CAPACITY and no sequence is live.  first_set_mask may then only keep layers whose
 * KV was stored for that sequence, and first_kv_read / first_kv_write refuse the others
 * (FIRST_ERR_STATE).  Results are bit-identical to a context without elision. */
int first_create(const first_model_desc *desc, const first_weights *weights, void *hip_stream,
                 first_ctx **out);
int first_destroy(first_ctx *ctx);

/* Prefill and route (Section 4.1, Section 4.3 item 1).  Drops any earlier sequences, then
 * for each of the B prompts runs ALL layers (no skipping), fills the KV cache of every
 * layer, evaluates router i on the stream entering layer i, fixes mask[b][i] =
 * (rho >= 0.5), compacts the kept-layer indices, and produces the first token from the
 * full model.  Synchronises the stream before returning (the masks are needed on the host).
 *   ids        DEV  int32 [sum(lens)]  prompts packed back to back
 *   lens       HOST int32 [B]          1 <= lens[b] < max_seq_len
 *   rho_out    DEV  fp32  [B, L]       router probabilities           (may be NULL)
 *   mask_out   DEV  uint8 [B, L]       1 = keep                       (may be NULL)
 *   hidden_out DEV  fp32  [B, D]       H_L of the last prompt token   (may be NULL)
 *   logits_out DEV  fp32  [B, V]       first-token logits             (may be NULL)
 *   token_out  DEV  int32 [B]          greedy first token, lowest index on ties (may be NULL) */
int first_prefill_route(first_ctx *ctx, int32_t B, const int32_t *ids, const int32_t *lens,
                        float *rho_out, uint8_t *mask_out, float *hidden_out,
                        float *logits_out, int32_t *token_out);

/* Benchmark override of the cached decisions of one sequence (this is how random-skip and
 * fixed-interval baselines of Section 5 are fed in).  Legal after prefill; once the
 * sequence has decoded a token only bits may be cleared, since re-enabling a layer would
 * leave holes in its KV (Section 4.3 item 2) -> FIRST_ERR_STATE.  mask: HOST uint8 [L]. */
int first_set_mask(first_ctx *ctx, int32_t seq, const uint8_t *mask);

/* Kept-layer indices of one sequence, ascending, as compacted on the device.
 * kept_idx HOST int32 [L], n_kept HOST int32 [1].  Synchronises the stream. */
int first_get_kept(first_ctx *ctx, int32_t seq, int32_t *kept_idx, int32_t *n_kept);

/* One decode token for every live sequence (Section 4.3 item 2; Section 3 rounded form):
 * h = E[token]; for each kept layer: RMSNorm, QKV, RoPE, KV append at position len[b],
 * GQA attention over positions 0..len[b], O projection, SwiGLU MLP; skipped layers are not
 * launched, leave h bit-identical and never touch their KV; then final norm, LM head and
 * greedy argmax.  len[b] grows by one.
 *   last_tokens DEV int32 [B]; logits_out DEV fp32 [B, V] (may be NULL); token_out DEV int32 [B].
 * FIRST_ERR_STATE before prefill, FIRST_ERR_CAPACITY when a sequence is full or no KV page is left (checked for
 * every sequence before any page is handed out: a refusal changes nothing).  The token ids live on the device, where
 * the host cannot see them: an id outside [0, vocab) is clamped to that range by the kernels, not refused. */
int first_decode_step(first_ctx *ctx, const int32_t *last_tokens, float *logits_out,
                      int32_t *token_out);

/* The decoding rule the paper times (Appendix, "Inference settings": temperature 0.8, top-k sampling
 * over 10 tokens) applied to the logits of the live sequences, e.g. those first_decode_step or
 * first_prefill_route just wrote: the candidates of a sequence are its top_k largest logits (equal
 * logits in order of token index), their weights exp((l - l_max) / temperature) are summed in
 * descending-logit order in fp32, and the token returned is the first candidate whose cumulative
 * weight exceeds u * total.  The draws are the caller's: the library owns no random number generator.
 *   logits         DEV fp32  [B, V]      B = number of live sequences
 *   uniforms       DEV fp32  [B]         one number in [0, 1) per sequence
 *   temperature    > 0;  1 <= top_k <= 64
 *   token_out      DEV int32 [B]         may be the buffer the next first_decode_step reads
 *   candidates_out DEV int32 [B, top_k]  the candidates in order, -1 beyond the vocabulary (may be NULL)
 * Enqueued on the context's stream.  FIRST_ERR_ARG on null pointers or parameters out of range,
 * FIRST_ERR_STATE when no sequence is live; nothing is written on error. */
int first_sample_top_k(first_ctx *ctx, const float *logits, const float *uniforms, float temperature,
                       int32_t top_k, int32_t *token_out, int32_t *candidates_out);

/* first_decode_step with that decoding rule in place of the greedy argmax (Appendix, "Inference settings"): the
 * token written for sequence b is drawn from its top_k largest logits exactly as first_sample_top_k would draw it
 * from the step's logits with the same uniforms (same candidates, same order, same fp32 arithmetic).  With one live
 * sequence on the persistent kernel the rule is part of that kernel: every workgroup lists the first top_k
 * candidates among its rows of the LM head and the workgroup that used to reduce the argmax merges the lists and
 * draws, so the step stays one launch and writes no logits unless asked to.  On the other decode paths, or when
 * top_k lists of all workgroups do not fit that kernel's LDS, the step's logits go through the kernels of
 * first_sample_top_k on the same stream (into a buffer of the context if logits_out is NULL).
 *   last_tokens DEV int32 [B]; uniforms DEV fp32 [B], one number in [0, 1) per sequence, read when the step runs;
 *   temperature > 0; 1 <= top_k <= 64; logits_out DEV fp32 [B, V] (may be NULL); token_out DEV int32 [B];
 *   candidates_out DEV int32 [B, top_k] (may be NULL).
 * Errors as first_decode_step and first_sample_top_k; a refusal changes nothing. */
int first_decode_step_sampled(first_ctx *ctx, const int32_t *last_tokens, const float *uniforms, float temperature,
                              int32_t top_k, float *logits_out, int32_t *token_out, int32_t *candidates_out);

/* first_sample_top_k for callers that cannot allocate device memory or hold a context: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same rule, same kernels and the same
 * results as first_sample_top_k, on any logits: the per-chunk candidate lists of the first stage live in a
 * 1 MiB device array that is part of the library image (one copy per GPU, held until the process ends), and
 * the call makes no hipMalloc / hipFree or other allocating call.
 *   hip_stream     hipStream_t the two kernels are enqueued on (NULL: the null stream)
 *   logits         DEV fp32  [n_seq, vocab]
 *   uniforms       DEV fp32  [n_seq]          one number in [0, 1) per sequence
 *   token_out      DEV int32 [n_seq]
 *   candidates_out DEV int32 [n_seq, top_k]   (may be NULL)
 * Limit: n_seq * ceil(vocab / 2048) * top_k <= 131072, else FIRST_ERR_CAPACITY (e.g. vocab 128256, top_k 10:
 * up to 208 sequences).  FIRST_ERR_ARG on null pointers or parameters out of range; nothing is written on
 * error; the text of the failure is first_last_error(NULL).  All calls on one GPU share that GPU's array:
 * calls that may overlap in time on one GPU (different streams, different threads) race and must be
 * serialised by the caller; calls on one stream are ordered and safe. */
int first_sample_top_k_static(void *hip_stream, const float *logits, int32_t n_seq, int32_t vocab,
                              const float *uniforms, float temperature, int32_t top_k,
                              int32_t *token_out, int32_t *candidates_out);

int first_set_option(first_ctx *ctx, int32_t option, int32_t value);
/* hipStreamSynchronize of the stream.  The workgroups of the persistent decode kernel wait for each other with bounded
 * waits; one that gives up (it should never happen: it means part of the grid was not running) makes every later
 * launch leave at its first wait, so tokens and logits stop changing.  first_sync - and every other entry point that
 * synchronises the stream: first_get_kept, first_seq_len, first_get_hidden, first_kv_read / first_kv_write - reports
 * this once as FIRST_ERR_HIP and resets the exchange state; the steps since the failed wait must be repeated. */
int first_sync(first_ctx *ctx);
const char *first_last_error(const first_ctx *ctx);      /* ctx may be NULL: last create error */

/* ---- inspection taps used by the parity tests (synchronise the stream) ------------------ */

/* Current length (prompt + decoded tokens) of a sequence and its number of live sequences. */
int first_seq_len(first_ctx *ctx, int32_t seq, int32_t *len_out /*HOST*/);
int first_batch(first_ctx *ctx, int32_t *batch_out /*HOST*/);

/* Gathers / scatters positions [pos0, pos0+n) of one layer's KV of one sequence through the
 * page table.  k, v: DEV fp32 [n, Hkv, hd] (values converted from / rounded to the KV type). */
int first_kv_read(first_ctx *ctx, int32_t seq, int32_t layer, int32_t pos0, int32_t n,
                  float *k_out, float *v_out);
int first_kv_write(first_ctx *ctx, int32_t seq, int32_t layer, int32_t pos0, int32_t n,
                   const float *k_in, const float *v_in);

/* Test tap: declares that sequence `seq` holds `len` tokens (1 <= len < max_seq_len), handing it the
 * pages that length needs.  The KV of positions the library never computed is whatever
 * first_kv_write put there (long-context checks on directly written KV).  Does not touch masks. */
int first_set_seq_len(first_ctx *ctx, int32_t seq, int32_t len);

/* Residual stream after the last decode step (before the final norm).  DEV fp32 [B, D]. */
int first_get_hidden(first_ctx *ctx, float *hidden_out);

/* Order in which free KV pages are handed out: perm HOST int32 [n_pages] a permutation of
 * 0..n_pages-1.  Legal only while no sequence is live.  n_pages via first_num_pages. */
int first_set_page_order(first_ctx *ctx, const int32_t *perm);
int first_num_pages(first_ctx *ctx, int32_t *n_pages_out /*HOST*/);

/* Size of the KV page pool and its layer slices (see first_create on elision).  All outputs
 * HOST, each may be NULL: pool_bytes = bytes allocated for KV pages (slots + scratch slice),
 * layer_slots = slices available to layers (n_layers without elision), slots_in_use = slices
 * handed to layers by the latest first_prefill_route (n_layers without elision). */
int first_kv_usage(first_ctx *ctx, int64_t *pool_bytes, int32_t *layer_slots, int32_t *slots_in_use);

/* ---- training-side forward pieces (forward values only: no gradients, no optimiser) ------- */

/* Soft-skip forward with the loss terms of router training (Section 4.1).  For each of the B
 * sequences every layer runs on the whole sequence, and its update enters the stream scaled by
 * the router's score of the stream that reached it: H_i = H_{i-1} + rho_i * phi_i(H_{i-1})
 * (the skip connection of the training figure read as an expectation; rounding rho_i gives
 * Eq. 2 of Section 3).  Then per sequence b:
 *   terms[b][0] = L_CE  : next-token cross entropy (natural log), mean over the positions j with
 *                         targets[j] >= 0, of the logits W_lm . RMSNorm(H_L[j]); 0 if none
 *   terms[b][1] = L_Reg : sum_i ||R_i||^2 over all router weights
 *   terms[b][2] = L_PP  : sum_i rho_i of this sequence
 *   terms[b][3] = L_CE + lambda * L_Reg + alpha * L_PP
 *   ids        DEV  int32 [sum(lens)]  sequences packed back to back
 *   lens       HOST int32 [B]          1 <= lens[b] <= max_seq_len
 *   targets    DEV  int32 [sum(lens)]  token to predict at each position, -1 = none
 *   rho_out    DEV  fp32  [B, L]       (may be NULL)
 *   terms_out  DEV  fp32  [B, 4]
 *   hidden_out DEV  fp32  [sum(lens), D]  H_L of every position (may be NULL)
 * Uses the context's prefill workspace and KV pages: any live sequences are dropped, and none
 * is live afterwards.  The first call allocates its workspace (one more stream copy, the
 * logits of 128 positions).  Synchronises the stream before returning. */
int first_soft_forward(first_ctx *ctx, int32_t B, const int32_t *ids, const int32_t *lens,
                       const int32_t *targets, float lambda, float alpha, float *rho_out,
                       float *terms_out, float *hidden_out);

/* LoRA merge (Section 4.2; appendix on the training set-up: rank 8, lora_alpha 32): in place
 * W += scale * Bm A with scale = lora_alpha / r, so that the adapters cost nothing at
 * inference.  W DEV [n, k] of dtype (row-major, as in first_weights); A DEV fp32 [r, k];
 * Bm DEV fp32 [n, r]; k multiple of 8; 1 <= r <= 32.  The rank-r sum is formed in fp32 in
 * index order and the result rounded once to dtype.  Asynchronous on hip_stream.  A context
 * created from W before the merge keeps what it copied (tile-order copies of batched decode):
 * merge first, then create. */
int first_lora_merge(void *hip_stream, int32_t dtype, void *W, const float *A, const float *Bm,
                     int32_t n, int32_t k, int32_t r, float scale);

/* ---- single fused ops, exposed for unit parity tests and kernel-level rooflines ---------- */

/* y[r] = sum_k W[r,k] * x[k]  (+ y_in[r] if accumulate).  The decode projection kernel.
 * W DEV [n, k] of dtype; x DEV fp32 [k]; y DEV fp32 [n]; k multiple of 8. */
int first_op_gemv(void *hip_stream, int32_t dtype, const void *W, const float *x, float *y,
                  int32_t n, int32_t k, int32_t accumulate);

/* C[m,n] = sum_k A[m,k] * W[n,k]  (+ C if accumulate).  The prefill projection kernel
 * (MFMA for bf16).  A DEV [m,k] and W DEV [n,k] of dtype, C DEV fp32 [m,n]; k multiple of 8. */
int first_op_gemm_nt(void *hip_stream, int32_t dtype, const void *A, const void *W, float *C,
                     int32_t m, int32_t n, int32_t k, int32_t accumulate);

/* The same contraction with fp32 activations and bf16 weights, as the prefill path runs it:
 * each activation is split into a high and a low bf16 part and both go through the matrix
 * cores, so about 16 bits of the activation's mantissa take part.
 * A DEV fp32 [m,k], W DEV bf16 [n,k], C DEV fp32 [m,n]; k multiple of 8. */
int first_op_gemm_nt_f32a(void *hip_stream, const float *A, const void *W, float *C, int32_t m,
                          int32_t n, int32_t k, int32_t accumulate);

/* Per-phase timestamps of the last persistent-kernel decode step (FIRST_OPT_STEP_TIMING = 1),
 * taken by workgroup 0 on the 100 MHz device clock: for each phase (QKV, O, gate/up, down of
 * every kept layer in order, then the LM head) twelve values: phase begins (twice), attention
 * done (O phase only), input staged, weights streamed, results stored, then six marks inside the
 * attention of workgroup 0 (O phase only): start, queries in LDS, tiles done, waves folded, other
 * splits' results arrived, output stored.  stamps HOST uint64 [capacity]; n_out HOST receives the
 * count.  Synchronises. */
int first_step_timing(first_ctx *ctx, uint64_t *stamps, int32_t capacity, int32_t *n_out);

/* Launches only the gate/up kernel of one layer (the largest kernel of a decode step,
 * Section 2 Eq. 1's phi_i: z = silu(Wg y) * (Wu y), y = RMSNorm(h)) for sequence slot seq, on
 * the context stream, reading the residual h[seq] and overwriting the MLP activation
 * workspace z[seq] (dead between decode steps).  For kernel-level timing. */
int first_op_gateup(first_ctx *ctx, int32_t layer, int32_t seq);

#ifdef __cplusplus
}
#endif
#endif /* FIRST_H_ */
