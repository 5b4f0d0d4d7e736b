/*
 * mace.h - C ABI of the MI355X hybrid-iteration library.
 *
 * One hybrid iteration of a pre-norm decoder layer over a mixed token batch: prefill rows,
 * decode rows (one per request, attending to a paged KV cache) and fine-tune rows (the two
 * sequences prompt+chosen / prompt+rejected of each preference pair) are processed by the same
 * launch sequence, followed by the DPO head and the backward pass of the fine-tune rows.  This
 * is what the executor of the paper's serving loop runs on the GPU for one scheduled bin
 * (Fig. 1, Section 4, Section 5); the scheduler that forms the bin is not part of this library.
 *
 * Conventions
 *  - "device" pointers are HIP device memory owned by the caller; "host" pointers are ordinary
 *    host memory.  The library never frees or keeps a caller pointer after a call returns.
 *  - All device work is ordered on the `stream` argument (a hipStream_t passed as void*, NULL =
 *    the default stream).  Calls do not synchronise with the host; outputs are valid once the
 *    caller has synchronised the stream.  Inside a call, products that nothing later in the call
 *    depends on (weight gradients, adapter products) may run on one internal stream of the handle,
 *    forked from `stream` and joined back into it with events before the call returns (also on
 *    every error return), so the caller sees plain stream order; MACE_OPT_SINGLE_STREAM keeps
 *    everything on `stream`.
 *  - A handle carries per-call state (the internal stream, its fork/join events, the launch-plan
 *    and timing records), so it supports ONE call in flight: calls on one handle must be issued
 *    from one thread at a time and on one stream (or on streams the caller has ordered against
 *    each other); use one handle per concurrent stream.  The three iteration calls of a step share
 *    the caller's workspace and must be issued in stream order.
 *  - Device memory: the caller owns every buffer.  The only device allocations of the library are
 *    made in mace_create (rotary frequency table, a few hundred bytes) and released in
 *    mace_destroy; no entry point allocates or frees device memory otherwise, and none issues a
 *    memset, so the iteration calls may be captured into a HIP graph.
 *  - Device-side descriptors (slots, block ids, labels, positions) are bounds-checked by the
 *    kernels: an out-of-range value never causes a wild access, but the affected row's result is
 *    then unspecified (see the preconditions at each entry point).
 *  - Every entry point returns MACE_OK (0) or a negative mace_status_t.  Arguments are validated
 *    on the host before anything is launched; mace_last_error() returns a message for the last
 *    failure on the calling thread.  No C++ exception crosses this boundary.
 *  - Matrices are row-major [out, in].  io_dtype selects the element type of x, the weights, the
 *    gains and the KV cache: MACE_BF16 (2-byte bfloat16) or MACE_F32.  Internal accumulation is
 *    fp32; y, all gradients, losses and log-probabilities are fp32.
 *  - Rows of the token batch are ordered prefill | decode | fine-tune.  Fine-tune sequence 2i is
 *    prompt+chosen of pair i, 2i+1 is prompt+rejected.
 */
#ifndef MACE_H
#define MACE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MACE_OK = 0,
  MACE_INVALID_ARG = -1,        /* null pointer, negative count, inconsistent offsets */
  MACE_BAD_SHAPE = -2,          /* model dimensions the kernels do not support */
  MACE_WORKSPACE_TOO_SMALL = -3,
  MACE_HIP_ERROR = -4           /* a HIP runtime call or launch failed */
} mace_status_t;

enum { MACE_F32 = 0, MACE_BF16 = 1 };

typedef struct mace_ctx *mace_handle_t;

/* Model dimensions.  Constraints (else MACE_BAD_SHAPE): head_dim is 64 or 128; n_q_heads /
 * n_kv_heads is 1, 2, 4 or 8; d_model (<= 8192), d_ff and vocab are multiples of 64. */
typedef struct {
  int32_t d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab;
  float rms_eps;       /* RMSNorm epsilon */
  float rope_theta;    /* rotary base; pair (i, i+head_dim/2) rotates by pos * theta^(-2i/head_dim) */
  int32_t io_dtype;    /* MACE_F32 or MACE_BF16 */
} mace_model_t;

/* Layer weights, device, io_dtype.  g_attn/g_mlp: RMSNorm gains [d_model].  wq [Hq*hd, d], wk and
 * wv [Hkv*hd, d], wo [d, Hq*hd], w_gate and w_up [d_ff, d], w_down [d, d_ff]. */
typedef struct {
  const void *g_attn, *wq, *wk, *wv, *wo, *g_mlp, *w_gate, *w_up, *w_down;
} mace_layer_w_t;

/* Gradients of the same tensors, device, fp32, same shapes.  Any pointer may be NULL (skipped). */
typedef struct {
  float *g_attn, *wq, *wk, *wv, *wo, *g_mlp, *w_gate, *w_up, *w_down;
} mace_layer_grads_t;

/* Paged KV cache (the PagedAttention-style cache of Section 5): K and V separately, each
 * [num_blocks, n_kv_heads, block_size, head_dim] in io_dtype, device.  K rows are stored after
 * the rotary embedding.  block_size is a power of two (1..256). */
typedef struct {
  void *k, *v;
  int64_t num_blocks;
  int32_t block_size;
} mace_kv_cache_t;

/* Batch descriptor of one iteration.  n_tokens = T_p + T_d + T_f with T_d = n_decode. */
typedef struct {
  int32_t n_prefill, n_decode, n_ft_seq, n_tokens;
  const int32_t *seg_offsets_host; /* host   [n_prefill+n_decode+n_ft_seq+1] first row of every request, last = n_tokens */
  const int32_t *seg_offsets;      /* device copy of the same array */
  const int32_t *positions;        /* device [n_tokens] rotary position of every row */
  const int32_t *slot_mapping;     /* device [T_p+T_d] cache slot of every inference row, -1 = do not store (prefill rows
                                      only: a decode row reads its own K, V back from the cache, so it must store them) */
  const int32_t *block_tables;     /* device [n_decode, max_blocks_per_req] block ids of the decode requests */
  const int32_t *context_lens_host;/* host   [n_decode] tokens already cached (the new token is not counted) */
  const int32_t *context_lens;     /* device copy of the same array */
  int32_t max_blocks_per_req;
  /* Prefix sharing (Section 4.3, "Reduced prefill via prefix tree"): prefill request i may have its
   * first prefill_prefix_lens[i] tokens cached already (K, V of a shared prefix node); its rows then
   * sit at positions prefix.., are appended behind the prefix (slot_mapping computed with
   * start_pos = prefix) and attend to the cached rows through prefill_block_tables[i], which
   * covers prefix + new tokens.  Requests below one node list the same leading blocks.  All three
   * pointers NULL = no request has a prefix.  Needs a bf16 cache (io_dtype MACE_BF16).
   * Precondition (not checkable here, block tables live on the device): a block that two requests of
   * one batch share must be full of prefix tokens, i.e. a shared prefix ends on a block boundary;
   * otherwise both requests append into that block. */
  const int32_t *prefill_block_tables;      /* device [n_prefill, max_blocks_per_prefill] */
  const int32_t *prefill_prefix_lens_host;  /* host   [n_prefill] */
  const int32_t *prefill_prefix_lens;       /* device copy of the same array */
  int32_t max_blocks_per_prefill;
  /* Shared-prompt preference pairs (the exact optimisation of the DPO forward/backward: a pair
   * (x, y+, y-) of Section 3.1 stored ONCE as the rows  prompt | chosen response | rejected response,
   * positions 0..P-1 | P.. | P..).  Fine-tune sequence s is then one pair; its rows at or beyond
   * ft_excl_hi[s] (the rejected response) do not attend to rows ft_excl_lo[s] .. ft_excl_hi[s]-1
   * (the chosen response); everything else is causal over the stored order.  Device int32
   * [n_ft_seq], row numbers relative to the sequence start; both NULL = ordinary sequences.
   * mace_dpo_logprob_loss_shared is the matching head. */
  const int32_t *ft_excl_lo, *ft_excl_hi;
  float *decode_head_norms;        /* optional OUTPUT, device fp32 [n_decode, n_q_heads]: L2 norm of every head's attention
                                      output vector of each decode row (before the output projection) - the signal of the
                                      norm-based cache pruning of Section 4.3; NULL = not wanted */
} mace_batch_t;

/* Create / destroy a handle for the device that is current at the call.  The handle owns a few
 * hundred bytes of device tables (rotary frequencies), one non-blocking stream of default priority
 * and ten events. */
int mace_create(mace_handle_t *out, const mace_model_t *model);
void mace_destroy(mace_handle_t h);

/* Options of a handle; every option is 0 after mace_create.  MACE_INVALID_ARG for an unknown option
 * or a value outside its range.  Set between calls, never while a call of the handle is in flight.
 *   MACE_OPT_HEAD_TWO_PASS  1: the DPO head forms every logit from two-term activations (two passes
 *                           over the vocabulary for bf16 weights); 0: the default head described
 *                           at mace_dpo_logprob_loss.
 *   MACE_OPT_SINGLE_STREAM  1: never use the internal stream (bitwise the same results).
 *   MACE_OPT_DECODE_CHUNK   tokens of context per decode-attention block: 0 = chosen per launch,
 *                           else a power of two in 512..4096.  The size of the partial-state scratch
 *                           depends on it: set it before mace_workspace_bytes is asked. */
enum { MACE_OPT_HEAD_TWO_PASS = 1, MACE_OPT_SINGLE_STREAM = 2, MACE_OPT_DECODE_CHUNK = 3 };
int mace_set_option(mace_handle_t h, int32_t option, int32_t value);

/* Message for the last error on this thread ("" if none). */
const char *mace_last_error(void);

/* Bytes of the buffer that carries fine-tune activations from the forward to the backward pass. */
size_t mace_fwd_saved_bytes(mace_handle_t h, int32_t n_ft_tokens);
/* Bytes of scratch the forward, backward and DPO calls need for a batch of these sizes
 * (n_tokens total rows, n_ft_tokens fine-tune rows, n_decode requests with at most
 * max_context cached tokens, n_loss_rows response tokens).  One workspace of this size serves
 * all three calls of an iteration; its contents need not survive between calls. */
size_t mace_workspace_bytes(mace_handle_t h, int32_t n_tokens, int32_t n_ft_tokens, int32_t n_decode,
                            int32_t max_context, int32_t n_loss_rows);

/* Host, pure integer: cache slots of positions start_pos .. start_pos+n-1 of one request,
 * slot(p) = block_table[p / B] * B + p % B (paged cache of Section 5).  table_len entries are
 * readable; MACE_INVALID_ARG if a position falls outside the table or an entry is negative. */
int mace_kv_slot_mapping(const int32_t *block_table, int32_t table_len, int32_t block_size,
                         int32_t start_pos, int32_t n, int32_t *slots_out);

/* Scatter n new rows k_new, v_new [n, Hkv, hd] (device, io_dtype) into the cache at
 * slot_mapping[n] (device; -1 or out-of-range slots are skipped).  "Only one token is appended
 * per iteration" per decode request (Section 3.2); prefill appends the whole prompt. */
int mace_kv_cache_append(mace_handle_t h, mace_kv_cache_t *cache, const void *k_new, const void *v_new,
                         const int32_t *slot_mapping, int32_t n, void *stream);

/* The read side of the paged cache of Section 5 (the engine's PagedAttention-style cache; "KV cache
 * accumulation" over the decode steps, Section 3.2): gather the rows of positions 0..ctx_len-1 of
 * one request, in order, into k_out, v_out [ctx_len, Hkv, hd] (device, io_dtype; bit-exact copies).  block_table: device
 * [ceil(ctx_len/B)].  slots_out: optional device int64 [ctx_len], the slot of every row. */
int mace_kv_cache_gather(mace_handle_t h, const mace_kv_cache_t *cache, const int32_t *block_table,
                         int32_t ctx_len, void *k_out, void *v_out, int64_t *slots_out, void *stream);

/* Forward of all rows of the iteration (Fig. 1: prefill, decode and fine-tune work colocated in
 * one iteration; every row sees the same weights).
 *   x  device [n_tokens, d_model] io_dtype;  y  device [n_tokens, d_model] fp32.
 * Prefill and decode rows write their post-rotary K and V to `cache` at slot_mapping; decode
 * rows attend to context_lens[r] cached tokens plus their own.  Fine-tune rows cache nothing;
 * their activations go to `saved` (mace_fwd_saved_bytes) for mace_hybrid_layer_bwd.
 * Fine-tune rows are computed with two-term bf16 operands (about 16 significand bits) so that
 * the DPO loss meets its 1e-3 tolerance; inference rows use plain bf16 operands.
 * Preconditions on device data: slots and block ids inside the cache, positions >= 0; a decode
 * row's slot_mapping entry is the slot of position context_lens[r] in its block table. */
int mace_hybrid_layer_fwd(mace_handle_t h, const mace_layer_w_t *w, const mace_batch_t *batch,
                          mace_kv_cache_t *cache, const void *x, float *y, void *saved,
                          void *workspace, size_t workspace_bytes, void *stream);

/* Backward of the fine-tune rows: the retraining half of the colocated iteration (Fig. 1 and
 * Section 3.2: the fine-tune worker's backward pass runs in the same iteration as prefill and decode;
 * Section 3.1: the gradient is that of the DPO objective, handed in as dy_ft).  Produces dL/dx of
 * the fine-tune rows and dL/dW of all seven matrices and both gains of the layer.
 * dy_ft device fp32 [T_f, d_model] (dL/dy of the fine-tune rows,
 * e.g. dh_ft of mace_dpo_logprob_loss); x the same x as in the forward; dx_ft device fp32
 * [T_f, d_model].  grads: fp32 weight gradients, summed over all fine-tune rows; overwritten, or
 * added to when accumulate != 0. */
int mace_hybrid_layer_bwd(mace_handle_t h, const mace_layer_w_t *w, const mace_batch_t *batch,
                          const void *x, const float *dy_ft, const void *saved, float *dx_ft,
                          const mace_layer_grads_t *grads, int accumulate,
                          void *workspace, size_t workspace_bytes, void *stream);

/* Adapter (LoRA) variant of the two layer calls (Section 5, fine-tune worker: every user or domain
 * owns a low-rank adapter while the base model stays frozen and shared by all requests).  The
 * four attention projections become  u W^T + scale * (u A^T) B^T  with A [rank, in] and
 * B [out, rank] (device, io_dtype, row-major; in/out as for wq, wk, wv, wo), 1 <= rank <= 64.
 * Every row of the iteration sees base + adapter.  The backward forms no base-weight gradient:
 * it returns dx_ft and the fp32 gradients of the eight adapter matrices (same shapes; a NULL
 * pointer skips that one; overwritten, or added to when accumulate != 0).  Workspace and saved
 * sizes are those of mace_workspace_bytes / mace_fwd_saved_bytes. */
typedef struct {
  const void *a_q, *b_q, *a_k, *b_k, *a_v, *b_v, *a_o, *b_o;
  int32_t rank;
  float scale;
} mace_lora_t;
typedef struct {
  float *a_q, *b_q, *a_k, *b_k, *a_v, *b_v, *a_o, *b_o;
} mace_lora_grads_t;
int mace_hybrid_layer_fwd_lora(mace_handle_t h, const mace_layer_w_t *w, const mace_lora_t *lora,
                               const mace_batch_t *batch, mace_kv_cache_t *cache, const void *x, float *y,
                               void *saved, void *workspace, size_t workspace_bytes, void *stream);
int mace_hybrid_layer_bwd_lora(mace_handle_t h, const mace_layer_w_t *w, const mace_lora_t *lora,
                               const mace_batch_t *batch, const void *x, const float *dy_ft,
                               const void *saved, float *dx_ft, const mace_lora_grads_t *grads,
                               int accumulate, void *workspace, size_t workspace_bytes, void *stream);

/* DPO head over the fine-tune rows (Section 3.1).  For sequence s with prompt length P_s and
 * length L_s, rows t = P_s-1 .. L_s-2 predict token t+1 through a final RMSNorm (gain g_final)
 * and the tied head w_lm [vocab, d_model]; log pi(y|x) is the sum of those log-probabilities.
 * Pair i: z = beta * ((logp[2i] - ref_logp[2i]) - (logp[2i+1] - ref_logp[2i+1])),
 * loss_per_pair[i] = -log sigmoid(z), loss_mean = mean over pairs.
 *   h_ft            device fp32 [T_f, d_model]  (rows of y of the fine-tune sequences)
 *   g_final, w_lm   device io_dtype
 *   token_ids       device int32 [T_f], every id in [0, vocab) (a label outside the range contributes
 *                   -logsumexp to its sequence and no one-hot term to the gradient)
 *   ft_seq_offsets  device and host int32 [n_seq+1], relative to the first fine-tune row
 *   prompt_lens     device and host int32 [n_seq]; 1 <= P_s <= L_s
 *   ref_logp        device fp32 [n_seq] (log pi_ref of each sequence, pre-computed)
 * Outputs (device fp32): logp_out [n_seq]; loss_per_pair [n_pairs]; loss_mean [1];
 *   clpd_out [n_pairs] = logp[2i]-logp[2i+1] (optional); win_out int32 [n_pairs] = clpd > 0 (optional).
 * Gradients of loss_mean (all optional, NULL = skipped; if all three are NULL no backward work is
 * done): dh_ft fp32 [T_f, d_model] (zero on rows that carry no loss), dw_lm fp32 [vocab, d_model]
 * (head contribution only), dg_final fp32 [d_model]; overwritten, or added to when accumulate != 0
 * (dh_ft is always overwritten).
 * Precision: the normalised rows n are held as two bf16 terms n_hi + n_lo (about 16 significand bits).
 * fp32 weights: every logit from two-term operands on both sides (three products).  bf16 weights, when a
 * gradient is requested: ONE pass over the vocabulary with n_hi, and the first-order effect of the dropped
 * n_lo on each row's log-probability, n_lo . (E_label - sum_j p_j E_j), is added back from the product
 * dlogits E that the backward forms anyway; the remainder is second order in n_lo (about 1e-7 per row).
 * bf16 weights without gradients, or with MACE_OPT_HEAD_TWO_PASS: two passes (n_hi, then n_lo). */
int mace_dpo_logprob_loss(mace_handle_t h, const float *h_ft, const void *g_final, const void *w_lm,
                          const int32_t *token_ids, const int32_t *ft_seq_offsets,
                          const int32_t *ft_seq_offsets_host, const int32_t *prompt_lens,
                          const int32_t *prompt_lens_host, int32_t n_pairs, const float *ref_logp,
                          float beta, float *logp_out, float *loss_per_pair, float *loss_mean,
                          float *clpd_out, int32_t *win_out, float *dh_ft, float *dw_lm,
                          float *dg_final, int accumulate, void *workspace, size_t workspace_bytes,
                          void *stream);

/* The same head for shared-prompt pairs (see mace_batch_t.ft_excl_lo): pair_offsets [n_pairs+1],
 * prompt_lens [n_pairs] and chosen_lens [n_pairs] (each as device and host array) describe stored
 * pair i = prompt (P_i rows) | chosen response (Rc_i rows) | rejected response.  The first token of
 * either response is predicted by the last prompt row, which therefore receives the gradient of
 * both.  logp_out / ref_logp keep the numbering 2i = chosen, 2i+1 = rejected; h_ft, dh_ft are
 * [sum of stored rows, d_model].  All other arguments as in mace_dpo_logprob_loss. */
int mace_dpo_logprob_loss_shared(mace_handle_t h, const float *h_ft, const void *g_final, const void *w_lm,
                                 const int32_t *token_ids, const int32_t *pair_offsets,
                                 const int32_t *pair_offsets_host, const int32_t *prompt_lens,
                                 const int32_t *prompt_lens_host, const int32_t *chosen_lens,
                                 const int32_t *chosen_lens_host, int32_t n_pairs, const float *ref_logp,
                                 float beta, float *logp_out, float *loss_per_pair, float *loss_mean,
                                 float *clpd_out, int32_t *win_out, float *dh_ft, float *dw_lm,
                                 float *dg_final, int accumulate, void *workspace, size_t workspace_bytes,
                                 void *stream);

/* Next-token logits of inference rows (decode rows, last row of a prefill request): what the
 * serving loop samples from and checks for end of sequence (Section 4.2, CheckEnd).  Row row_idx[i]
 * of y (device fp32 [*, d_model], the output of mace_hybrid_layer_fwd; row_idx device int32 [n],
 * NULL = rows 0..n-1) goes through the final RMSNorm (g_final) and the tied head w_lm [vocab, d]:
 * logits_out device fp32 [n, vocab] (required), next_token device int32 [n] (optional) = greedy
 * arg max of the fp32 logits, lowest index on ties.  Plain bf16 operands (inference precision).
 * Workspace: mace_workspace_bytes. */
int mace_next_token_logits(mace_handle_t h, const float *y, const int32_t *row_idx, int32_t n, const void *g_final,
                           const void *w_lm, float *logits_out, int32_t *next_token, void *workspace,
                           size_t workspace_bytes, void *stream);

/* mace_next_token_logits for callers that cannot allocate device memory or bring a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * without the workspace, same kernels, bit-identical results; the normalised rows go to a buffer
 * built into the library (4 MiB of device memory per GPU, held until the process ends) instead.
 * Limits: a bf16 model (MACE_BAD_SHAPE otherwise: fp32 weights would need a converted copy of the
 * head), n * d_model * 2 <= 4 MiB, e.g. 512 rows at d_model 4096 (MACE_WORKSPACE_TOO_SMALL
 * otherwise), and the device of mace_create must be current (MACE_INVALID_ARG otherwise).  The call
 * allocates and frees nothing and issues no memset.  Every call on one GPU, from any handle, shares
 * the one buffer: calls that overlap on a GPU (two streams, two threads) race; order them. */
int mace_next_token_logits_static(mace_handle_t h, const float *y, const int32_t *row_idx, int32_t n, const void *g_final,
                                  const void *w_lm, float *logits_out, int32_t *next_token, void *stream);

/* AdamW step (decoupled weight decay) on one tensor of n elements: the optimizer step that turns
 * the gradients of an iteration into the weights the next iteration sees (Section 2.1).  The paper
 * names no optimizer; AdamW is the reading.  step counts from 1.
 *   m <- b1 m + (1-b1) g ;  v <- b2 v + (1-b2) g^2
 *   p <- p - lr * ( (m / (1-b1^step)) / (sqrt(v / (1-b2^step)) + eps) + weight_decay * p )
 * param: device, the handle's io_dtype, updated in place.  master: optional device fp32 copy of the
 * parameter; when given it is the value that is updated and param is its rounding (for bf16 models;
 * without it a bf16 param is updated from its own rounded value).  grad, m, v device fp32.  All
 * pointers 16-byte aligned. */
int mace_adamw_step(mace_handle_t h, void *param, float *master, const float *grad, float *m, float *v, int64_t n,
                    float lr, float beta1, float beta2, float eps, float weight_decay, int32_t step, void *stream);

/* Cache-pruning statistics of Section 4.3 ("Decode KV cache pruning").
 * mace_head_norm_stats (device, elementwise over n requests x n_heads heads), given the norms of
 * this iteration (decode_head_norms of the forward):
 *   abar[r,h]  <-  abar[r,h] + (norm[r,h] - abar[r,h]) / t_count[r]     running mean over the t_count[r] decode
 *                                                                       iterations request r has had, this one included
 *   prune[r,h]  =  (t_count[r] - last_used[r,h] > window)  or  (norm[r,h] < tau)
 *   last_used[r,h]  <-  t_count[r] where norm[r,h] >= tau                (reading: "last used" = last iteration at
 *                                                                       which the head's norm reached tau)
 * abar fp32 in/out, t_count int32 (every entry >= 1; an entry < 1 leaves that request's abar, last_used
 * and prune untouched), last_used int32 in/out and prune int32 out (0/1) are device
 * arrays; last_used and prune may both be NULL (running mean only).
 * mace_kv_head_budget (host, pure): w_h = abar_h / sum_j abar_j, C_h = floor(w_h * c_total) in
 * double precision, and what the floors leave over goes one unit each to the heads of largest w_h
 * (ties: lower index first); sum_h c_out[h] == c_total.  abar must be positive and finite. */
int mace_head_norm_stats(mace_handle_t h, const float *norms, const int32_t *t_count, int32_t n, int32_t n_heads,
                         float *abar, int32_t *last_used, int32_t window, float tau, int32_t *prune, void *stream);
int mace_kv_head_budget(const double *abar, int32_t n_heads, int64_t c_total, int64_t *c_out);

/* Instrumentation for benchmarks (not part of the paper's method).  When enabled, every kernel
 * launch of the three iteration calls is preceded by a HIP event recorded on the call's stream
 * and each call ends with one more, so launch i lasts event[i+1] - event[i] on that stream.
 * mace_profile_collect waits for the last event (host-synchronising), sums launches, milliseconds
 * and algorithmic flops per kernel class into out[0 .. *n_out) (max_entries >= 16), and clears
 * the record.  At most 32768 launches are recorded between two collects; later ones are not timed.
 * on = 0: off; on = 1: every kernel class; any other value: bit (i + 1) selects class i of the
 * order in which mace_profile_collect reports them, and only launches of the selected classes are
 * bracketed (an event before the launch, one before whatever is launched next), which keeps the
 * cost of the events out of a timed region that needs one class only.  Launches that the
 * library puts on its internal side stream (weight-gradient and adapter GEMMs) are timed on that
 * stream and reported as classes of their own ("gemm_tn@side", ...; selected by the bit of the
 * plain class); they overlap with the main chain, so class times can add up to more than the
 * wall time and a side class does not show the speed of a kernel that has the chip to itself. */
typedef struct {
  char name[48];      /* kernel class: gemm_nt, gemm_nn, gemm_tn, attn_fwd_prefill, attn_fwd_ft, attn_decode, ... */
  int64_t launches;
  int64_t side_launches;  /* how many of them ran on the library's side stream, overlapping the main chain */
  double ms;          /* summed duration */
  double flops;       /* summed algorithmic flops (GEMM classes: 2*M*N*K once per launch, extra operand passes not counted) */
  double bytes;       /* summed algorithmic bytes where the class is HBM-bound, else 0 */
} mace_profile_entry_t;
int mace_profile_enable(mace_handle_t h, int on);
int mace_profile_collect(mace_handle_t h, mace_profile_entry_t *out, int32_t max_entries, int32_t *n_out);

/* Launch plan of the dense contractions (host-side record, for tests and benchmarks; not part of the
 * paper's method).  Every iteration call clears the record of the handle and then notes, for each
 * GEMM it launches in order, the decisions its launcher took from the problem sizes: block tile,
 * number of k slices, and whether the product ran on the internal stream.  A test at a reduced batch
 * compares these with the full-size launch to show that it exercises the same code path. */
typedef struct {
  char name[32];           /* which product: "qkv gemm", "dWd gemm", ... */
  int32_t layout;          /* 0 = NT (x W^T), 1 = NN (dy W), 2 = TN (dy^T x) */
  int32_t tile_m, tile_n;  /* block tile */
  int32_t k_splits;        /* k slices (1 = none) */
  int32_t on_side_stream;  /* 1 = issued on the internal stream */
  int64_t m, n, k;         /* rows summed over row groups, columns summed over segments, reduction length */
} mace_gemm_plan_t;
int mace_launch_plan(mace_handle_t h, mace_gemm_plan_t *out, int32_t max_entries, int32_t *n_out);

/* The dense contraction kernel on its own (for kernel-level tests and benchmarks; every product of the
 * iteration of Section 2.1 / Fig. 4 goes through the same launcher with the same operand forms).
 *   C[m, n] = sum_k A[m, k] B[n, k]  (+ sum_k A_lo[m, k] B[n, k])  (+ R[m, n])
 * A, A_lo, B: device bf16.  layout_a = 0: A is [M, K] row-major, 1: [K, M] row-major; layout_b = 0: B is [N, K]
 * row-major, 1: [K, N] row-major (supported pairs: (0,0), (0,1), (1,1)); lda, ldb, ldc, ldr in elements.  a_lo
 * (nullable) is the second bf16 term of A: given, the product takes two passes.  C: device, fp32 (out_bf16 = 0)
 * or bf16 (1), [M, N] with row stride ldc.  R (nullable): device fp32 (resid_kind = 1) or bf16 (2), row stride ldr.
 * swiglu = 1 (layouts (0,0) only): b holds the gate rows and b_up the up rows of N hidden units, and instead of
 * the products G and U the call writes hm = silu(G) * U as bf16 into c ([M, N], ldc), its second bf16 term
 * into c_lo (nullable) and G | U as bf16 [M, 2N] into c_gu (nullable).
 * swiglu = 2 (layouts (0,1), kernel = 1 only): the backward form.  The product is dHm [M, N]; c_gu holds G | U of the
 * forward (bf16 [M, 2N], read only) and instead of dHm the call writes dG | dU as bf16 [M, 2N] into c (ldc = 2N):
 * dG = dHm U s (1 + G (1 - s)), dU = dHm G s, s = sigmoid(G).
 * rope_cs != NULL (layouts (0,0), kernel = 1 only, N a multiple of 128): the rotary form of the QKV product.  The
 * columns are heads of 128; rope_cs is a device fp32 table [M, 64, 2] of (cos, sin) per row and pair index.  Instead
 * of C the call writes the product as two bf16 terms, c (first) and c_lo (second, nullable), both [M, N] with row
 * stride N, after rotating every head (rope_rotate = 1: column i < 64 of a head becomes a cos - b sin and column i + 64
 * becomes b cos + a sin, a and b being the two columns' products) or unrotated (rope_rotate = 0).
 * kernel = 0: the launcher picks tile and kernel from the sizes as it does inside the iteration; 1: the 256x256
 * four-wave kernel (MACE_BAD_SHAPE where the problem does not fit it).
 * Requirements: K a multiple of 64 for a k-contiguous operand; M (N) a multiple of 8 for an m- (n-) contiguous
 * one; leading dimensions multiples of 8; pointers 16-byte aligned.  Nothing is allocated; the call is
 * asynchronous on `stream`.  Errors: MACE_INVALID_ARG (null pointers), MACE_BAD_SHAPE (the requirements). */
typedef struct {
  int32_t layout_a, layout_b;
  int32_t M, N, K;
  int64_t lda, ldb, ldc, ldr;
  const void *a, *a_lo, *b, *b_up;
  void *c, *c_lo, *c_gu;
  const void *resid;
  int32_t out_bf16, resid_kind, swiglu, kernel;
  const float *rope_cs;
  int32_t rope_rotate;
} mace_gemm_desc_t;
int mace_gemm_bf16(mace_handle_t h, const mace_gemm_desc_t *d, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MACE_H */
