// Host-callable launchers of the non-GEMM kernels.  All pointers are device pointers.
// Every launcher returns the HIP launch status.  "hi"/"lo" are the two bf16 terms of a value
// (lo pointers may be null: then only the rounded value is written).
#pragma once
#include "common.h"

// ---- elementwise.hip -------------------------------------------------------------------------
// Row-wise RMSNorm: out = x * rsqrt(mean(x^2) + eps) * g.  x is fp32 or bf16 [*, d] (row r reads
// input row row_idx[r] when row_idx is non-null), g is fp32 or bf16 [d].  rstd (nullable) gets
// the row scale.
hipError_t launch_rmsnorm_fwd(const void *x, bool x_bf16, const int32_t *row_idx, const void *g, bool g_bf16,
                              int rows, int d, float eps, bf16_t *hi, bf16_t *lo, float *rstd, hipStream_t st);
// RMSNorm backward.  dx_out[out_row] = resid[r] + rstd*(dy*g) - x*rstd^3*mean((dy*g)*x), where
// out_row = row_idx ? row_idx[r] : r and x is read at the same row; resid (nullable) fp32.
// dg_partial [n_part, d] receives per-block partial sums of dy*x*rstd (reduce with
// launch_colsum).  dx_bf (nullable) gets a bf16 copy of dx_out rows (same row mapping).
// dense_out != 0: output row r is written at row r (dx_out may then be dy itself) while x is still
// read at row_idx[r].
hipError_t launch_rmsnorm_bwd(const float *dy, const void *x, bool x_bf16, const int32_t *row_idx, const void *g,
                              bool g_bf16, const float *rstd, const float *resid, int rows, int d,
                              float *dx_out, bf16_t *dx_bf, float *dg_partial, int n_part, hipStream_t st,
                              int dense_out = 0);
// out[j] (+)= sum over the n_part rows of part[:, j]; scratch: COLSUM_SLICES * d floats.
constexpr int COLSUM_SLICES = 32;
hipError_t launch_colsum(const float *part, int n_part, int d, float *scratch, float *out, int accumulate, hipStream_t st);
// Rotary embedding of q and k inside qkv fp32 [rows, (Hq+2Hkv)*hd], split into head-major bf16
// outputs q [rows, Hq*hd], k, v [rows, Hkv*hd]; optionally scatter k, v (rounded to the cache
// type) into the paged cache at slot_mapping (null = no cache write).
hipError_t launch_rope_split(const float *qkv, const int32_t *positions, const double *inv_freq, int rows, int Hq,
                             int Hkv, int hd, bf16_t *q_hi, bf16_t *k_hi, bf16_t *v_hi, bf16_t *q_lo, bf16_t *k_lo,
                             bf16_t *v_lo, const int32_t *slot_mapping, void *cache_k, void *cache_v, bool cache_bf16,
                             long long num_slots, int block_size, hipStream_t st);
// cs[r, i] = (cos, sin) of positions[r] * inv_freq[i], i < hd/2 (angle formed and reduced in fp64): the
// per-row rotary table the attention backward rotates dq and dk back with.
hipError_t launch_rope_table(const int32_t *positions, const double *inv_freq, int rows, int hd, float2 *cs, hipStream_t st);
// dU = dhm*silu(G), dG = dhm*U*sig(G)*(1+G*(1-sig(G))) -> dgu bf16 [rows, 2F].
// gu bf16 [rows, 2F] (G = columns [0,F), U = [F,2F)) as the gate/up GEMM left it.  F % 8 == 0.
hipError_t launch_swiglu_bwd(const bf16_t *dhm, const bf16_t *gu, int rows, int F, bf16_t *dgu, hipStream_t st);
// fp32 -> (hi, lo) bf16, n elements; lo nullable.
hipError_t launch_split_f32(const float *src, size_t n, bf16_t *hi, bf16_t *lo, hipStream_t st);
hipError_t launch_fill_f32(float *dst, size_t n, float v, hipStream_t st);
// out[i] = sum_s part[s * n + i], n % 4 == 0 (partial sums of a split-K GEMM, fixed order).
hipError_t launch_sum_partials(const float *part, int n_part, size_t n, float *out, hipStream_t st);

// ---- lora.hip ---------------------------------------------------------------------------------
// dst[dst_rows, dst_cols] as bf16 (hi, nullable lo) = zeros with up to three source matrices
// (fp32 or bf16, [rows, cols] row-major), multiplied by scale, placed at (r0, c0).
hipError_t launch_lora_pack(const void *const *src, const int *rows, const int *cols, const int *r0, const int *c0, int n_src,
                            bool src_bf16, int dst_rows, int dst_cols, float scale, bf16_t *hi, bf16_t *lo, hipStream_t st);
// (hi, lo) = two-term bf16 form of scale * src.
hipError_t launch_scale_split(const float *src, size_t n, float scale, bf16_t *hi, bf16_t *lo, hipStream_t st);
// dst[rows, cols] (+)= scale * the window of src (row pitch src_ld) that starts at (r0, c0).
hipError_t launch_extract(const float *src, int src_ld, int r0, int c0, int rows, int cols, float scale, float *dst, int accumulate, hipStream_t st);

// ---- loop.hip ---------------------------------------------------------------------------------
// out[r] = arg max_j logits[r, j] (lowest index on ties), fp32 logits [rows, V].
hipError_t launch_argmax_rows(const float *logits, int rows, int V, int32_t *out, hipStream_t st);
// AdamW with decoupled weight decay on n elements; param in fp32 or bf16, master (nullable) the
// fp32 copy that is updated and from which param is rounded; c1, c2 = 1/(1-b1^t), 1/(1-b2^t).
hipError_t launch_adamw(void *param, bool param_bf16, float *master, const float *grad, float *m, float *v, size_t n, float lr,
                        float b1, float b2, float eps, float wd, float c1, float c2, hipStream_t st);

// ---- kv_cache.hip ----------------------------------------------------------------------------
hipError_t launch_kv_append(void *cache_k, void *cache_v, bool bf16, long long num_slots, int block_size, int Hkv,
                            int hd, const void *k_new, const void *v_new, const int32_t *slot_mapping, int n,
                            hipStream_t st);
hipError_t launch_kv_gather(const void *cache_k, const void *cache_v, bool bf16, long long num_blocks, int block_size,
                            int Hkv, int hd, const int32_t *block_table, int ctx_len, void *k_out, void *v_out,
                            long long *slots_out, hipStream_t st);

// ---- attn_fwd.hip ----------------------------------------------------------------------------
// Varlen causal attention over n_seq sequences.  seg points at n_seq+1 row offsets (device)
// ABSOLUTE in the batch; row_base is subtracted to index q/k/v/o (which start at the first row
// of this class).  lse (nullable) fp32 [rows, Hq].  split: operands are (hi, lo) pairs.
hipError_t launch_attn_fwd(const bf16_t *q_hi, const bf16_t *k_hi, const bf16_t *v_hi, const bf16_t *q_lo,
                           const bf16_t *k_lo, const bf16_t *v_lo, const int32_t *seg, int row_base, int n_seq,
                           int max_len, int Hq, int Hkv, int hd, bf16_t *o_hi, bf16_t *o_lo, float *lse,
                           hipStream_t st, const int32_t *excl_lo = nullptr, const int32_t *excl_hi = nullptr);
// excl_lo / excl_hi (nullable, device [n_seq], rows relative to the sequence start): queries at or
// beyond excl_hi[s] do not see keys excl_lo[s] .. excl_hi[s]-1 (shared-prompt preference pairs).
// The same for requests with a cached prefix: keys and values of request s are positions
// 0 .. prefix_lens[s] + len_s - 1 of its block table in the paged bf16 cache (its own rows must have
// been appended already); query j of the request sits at position prefix_lens[s] + j.
hipError_t launch_attn_fwd_paged(const bf16_t *q, const void *cache_k, const void *cache_v, long long num_blocks, int block_size,
                                 const int32_t *block_tables, int max_blocks, const int32_t *prefix_lens, const int32_t *seg,
                                 int row_base, int n_seq, int max_len, int Hq, int Hkv, int hd, bf16_t *o, hipStream_t st);
// ---- attn_decode.hip -------------------------------------------------------------------------
// One query row per request against its paged context of ctx_len[r]+1 tokens.  q bf16
// [n_decode, Hq*hd] (rows of the decode class), out bf16 same shape.  partial: fp32 scratch of
// decode_partial_floats() floats.  norms (nullable): fp32 [n_decode, Hq], L2 norm of each head's output.
size_t decode_partial_floats(int n_decode, int Hq, int Hkv, int hd, int max_context, int chunk_tokens);
hipError_t launch_attn_decode(const bf16_t *q, const void *cache_k, const void *cache_v, bool cache_bf16,
                              long long num_blocks, int block_size, const int32_t *block_tables, int max_blocks_per_req,
                              const int32_t *ctx_lens, int n_decode, int max_context, int Hq, int Hkv, int hd,
                              float *partial, bf16_t *out, float *norms, hipStream_t st, int chunk_tokens = 0);
// chunk_tokens: context tokens per block, 0 = chosen from the grid size, else a power of two in 512..4096.
// Running mean of the head norms, prune predicate and last-used bookkeeping (elementwise, n x H).
hipError_t launch_head_norm_stats(const float *norms, const int32_t *t_count, int n, int H, float *abar, int32_t *last_used,
                                  int window, float tau, int32_t *prune, hipStream_t st);
// ---- attn_bwd.hip ----------------------------------------------------------------------------
// Backward of the varlen causal attention of the fine-tune sequences (bf16 operands), rotary backward
// included: dqkv bf16 [rows, (Hq+2Hkv)*hd] receives dq and dk rotated back by the rows' angles (cs: the
// table of launch_rope_table, [rows, hd/2]) and dv, i.e. the gradient of the projection output.
// dvec: fp32 scratch [rows, Hq] (rowsum(dO * O), written by the dq kernel, read by the dk/dv kernel).
hipError_t launch_attn_bwd(const bf16_t *q, const bf16_t *k, const bf16_t *v, const bf16_t *o, const bf16_t *d_o,
                           const float *lse, const int32_t *seg, int row_base, int n_seq, int max_len, int rows,
                           int Hq, int Hkv, int hd, float *dvec, const float2 *cs, bf16_t *dqkv, hipStream_t st,
                           const int32_t *excl_lo = nullptr, const int32_t *excl_hi = nullptr);

// ---- dpo_head.hip ----------------------------------------------------------------------------
// For every loss row (sequence s, t = P_s-1 .. L_s-2, in sequence order): row_idx = index of row
// t among the fine-tune rows, label = token_ids[t+1], seq_id = s.
hipError_t launch_loss_rows(const int32_t *ft_seq_offsets, const int32_t *prompt_lens, const int32_t *token_ids,
                            int n_seq, int32_t *row_idx, int32_t *label, int32_t *seq_id, hipStream_t st);
// Shared-prompt layout (a pair stored once as prompt | chosen | rejected; offsets per PAIR): loss
// rows of sequence 2i (chosen) are the last prompt row and the chosen rows but the last, of 2i+1 the
// last prompt row and the rejected rows but the last.  partner[r]: -1, or for the chosen sequence's
// first loss row the index of the rejected sequence's first loss row (same target row), which
// itself gets -2.  vseq_off [2 n_pairs + 1] / vprompt [2 n_pairs]: a virtual (offsets, prompt
// lengths) pair with the loss-row counts of the 2 n_pairs sequences, for launch_dpo_pairs.
hipError_t launch_loss_rows_shared(const int32_t *pair_offsets, const int32_t *prompt_lens, const int32_t *chosen_lens,
                                   const int32_t *token_ids, int n_pairs, int32_t *row_idx, int32_t *label, int32_t *seq_id,
                                   int32_t *partner, int32_t *vseq_off, int32_t *vprompt, hipStream_t st);
// dst[row_idx[r], :] = src[r, :] (+ src[partner[r], :] when partner[r] >= 0); rows with partner -2 are skipped.
hipError_t launch_scatter_rows(const float *src, const int32_t *row_idx, const int32_t *partner, int rows, int d, float *dst,
                               hipStream_t st);
// logp_t[r] = logits[r, label[r]] - logsumexp(logits[r, :]); lse[r] kept.  dl (nullable) bf16 [rows, V]:
// dl[r, j] = [j == label[r]] - exp(logits[r, j] - lse[r]), the gradient of log p(label) with respect to the
// logits of the row, without the factor of the row's sequence (see launch_scale_rows).  V % 4 == 0.
hipError_t launch_logsoftmax_dl(const float *logits, int rows, int V, const int32_t *label, float *logp_t, float *lse, bf16_t *dl,
                               hipStream_t st);
// logp_t[r] += n_lo[r, :] . u[r, :]  (first-order term of a head that formed its logits from n_hi alone; u = dl E)
hipError_t launch_logp_correct(const bf16_t *n_lo, const float *u, int rows, int d, float *logp_t, hipStream_t st);
// c = dlogp[seq_id[r]]:  u[r, :] *= c (u nullable);  n_c[r, :] = bf16(c * n_hi[r, :]) (n_c nullable)
hipError_t launch_scale_rows(float *u, const bf16_t *n_hi, bf16_t *n_c, const int32_t *seq_id, const float *dlogp, int rows, int d,
                             hipStream_t st);
// Per-sequence sums, pair losses, metrics and dloss_mean/dlogp per sequence.
hipError_t launch_dpo_pairs(const float *logp_t, const int32_t *ft_seq_offsets, const int32_t *prompt_lens, int n_seq,
                            const float *ref_logp, float beta, float *logp_out, float *loss_per_pair, float *loss_mean,
                            float *clpd, int32_t *win, float *dlogp, hipStream_t st);
