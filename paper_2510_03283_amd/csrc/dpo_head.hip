// DPO head kernels (Section 3.1 of the paper): loss-row bookkeeping, vocabulary log-soft-max with
// label gather, per-sequence sums, pairwise sigmoid loss and the gradient of the logits.
#include "kernels.h"

namespace {

// One block per fine-tune sequence.  Loss rows of sequence s are t = P_s-1 .. L_s-2; their
// position in the packed list is the sum of (L_i - P_i) over the sequences before s.
__global__ __launch_bounds__(256) void loss_rows_kernel(const int32_t *ft_seq_offsets, const int32_t *prompt_lens,
                                                        const int32_t *token_ids, int32_t *row_idx, int32_t *label,
                                                        int32_t *seq_id) {
  const int s = blockIdx.x;
  int base = 0;
  for (int i = 0; i < s; ++i) base += (ft_seq_offsets[i + 1] - ft_seq_offsets[i]) - prompt_lens[i];
  const int o = ft_seq_offsets[s], L = ft_seq_offsets[s + 1] - o, P = prompt_lens[s];
  for (int i = threadIdx.x; i < L - P; i += 256) {
    const int t = P - 1 + i;
    row_idx[base + i] = o + t;
    label[base + i] = token_ids[o + t + 1];
    seq_id[base + i] = s;
  }
}

// Shared-prompt layout, one block per pair.
__global__ __launch_bounds__(256) void loss_rows_shared_kernel(const int32_t *pair_offsets, const int32_t *prompt_lens,
                                                               const int32_t *chosen_lens, const int32_t *token_ids, int n_pairs,
                                                               int32_t *row_idx, int32_t *label, int32_t *seq_id, int32_t *partner,
                                                               int32_t *vseq_off, int32_t *vprompt) {
  const int i = blockIdx.x;
  int base = 0;
  for (int k = 0; k < i; ++k) base += (pair_offsets[k + 1] - pair_offsets[k]) - prompt_lens[k];
  const int o = pair_offsets[i], L = pair_offsets[i + 1] - o, P = prompt_lens[i], Rc = chosen_lens[i], Rr = L - P - Rc;
  for (int q = 0; q < 2; ++q) {
    const int start = q ? P + Rc : P, R = q ? Rr : Rc, b0 = base + (q ? Rc : 0);
    for (int j = threadIdx.x; j < R; j += 256) {
      const int t = j == 0 ? P - 1 : start + j - 1;           // the row that predicts response token j
      row_idx[b0 + j] = o + t;
      label[b0 + j] = token_ids[o + start + j];
      seq_id[b0 + j] = 2 * i + q;
      partner[b0 + j] = j == 0 ? (q ? -2 : (Rr > 0 ? base + Rc : -1)) : -1;
    }
  }
  if (threadIdx.x == 0) {
    vseq_off[2 * i] = base;
    vseq_off[2 * i + 1] = base + Rc;
    if (i == n_pairs - 1) vseq_off[2 * n_pairs] = base + Rc + Rr;
    vprompt[2 * i] = vprompt[2 * i + 1] = 0;
  }
}

__global__ __launch_bounds__(256) void scatter_rows_kernel(const float *__restrict__ src, const int32_t *__restrict__ row_idx,
                                                           const int32_t *__restrict__ partner, int d, float *__restrict__ dst) {
  const int r = blockIdx.x, p = partner[r];
  if (p == -2) return;
  const float *a = src + (size_t)r * d, *b = p >= 0 ? src + (size_t)p * d : nullptr;
  float *o = dst + (size_t)row_idx[r] * d;
  for (int k = 4 * threadIdx.x; k < d; k += 1024) {        // d % 4 == 0
    float4 v = *(const float4 *)(a + k);
    if (b) { const float4 w = *(const float4 *)(b + k); v.x += w.x; v.y += w.y; v.z += w.z; v.w += w.w; }
    *(float4 *)(o + k) = v;
  }
}

// The logit of the label, recomputed from the two-term activations: one wave per loss row forms
// sum_k (n_hi + n_lo)[r, k] * E[label, k] in fp32 and overwrites logits[r, label].  With it the LM
// head runs one bf16 pass: the rounding of n to bf16 moves every logit of a row by a few 1e-4, which
// the log-sum-exp averages out (it enters as the rounding error times the soft-max mean of the
// embeddings), but which would enter the label's own logit - and so log p(label) - at full size.
__global__ __launch_bounds__(256) void label_logit_kernel(const bf16_t *__restrict__ n_hi, const bf16_t *__restrict__ n_lo,
                                                          const bf16_t *__restrict__ e, const int32_t *__restrict__ label,
                                                          int rows, int d, int V, float *__restrict__ logits) {
  const int lane = threadIdx.x & 63, r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const int lab = label[r];
  if (lab < 0 || lab >= V) return;
  const bf16_t *a = n_hi + (size_t)r * d, *b = n_lo + (size_t)r * d, *w = e + (size_t)lab * d;
  float s = 0.f;
  for (int k = lane * 8; k < d; k += 512) {        // d % 8 == 0
    const uint4 ua = *(const uint4 *)(a + k), ub = *(const uint4 *)(b + k), uw = *(const uint4 *)(w + k);
    const uint32_t wa[4] = {ua.x, ua.y, ua.z, ua.w}, wb[4] = {ub.x, ub.y, ub.z, ub.w}, ww[4] = {uw.x, uw.y, uw.z, uw.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      s += (__uint_as_float(wa[i] << 16) + __uint_as_float(wb[i] << 16)) * __uint_as_float(ww[i] << 16);
      s += (__uint_as_float(wa[i] & 0xffff0000u) + __uint_as_float(wb[i] & 0xffff0000u)) * __uint_as_float(ww[i] & 0xffff0000u);
    }
  }
  s = wave_sum(s);
  if (lane == 0) logits[(size_t)r * V + lab] = s;
}

// One block per loss row: single pass over the V logits with an online (max, sum) pair.
__global__ __launch_bounds__(256) void logsoftmax_gather_kernel(const float *__restrict__ logits, int V,
                                                                const int32_t *__restrict__ label,
                                                                float *__restrict__ logp_t, float *__restrict__ lse) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  const float *row = logits + (size_t)r * V;
  float m = -INFINITY, s = 0.f;
  for (int k = 4 * threadIdx.x; k < V; k += 1024) {       // V % 4 == 0
    const float4 v = *(const float4 *)(row + k);
    const float mx = fmaxf(fmaxf(v.x, v.y), fmaxf(v.z, v.w));
    if (mx > m) { s *= expf(m - mx); m = mx; }
    s += expf(v.x - m) + expf(v.y - m) + expf(v.z - m) + expf(v.w - m);
  }
  const float mb = block_max<256>(m, red);
  s = (m == -INFINITY) ? 0.f : s * expf(m - mb);
  const float sb = block_sum<256>(s, red);
  if (threadIdx.x == 0) {
    const float l = mb + logf(sb);
    lse[r] = l;
    const int lab = label[r];
    logp_t[r] = (lab >= 0 && lab < V ? row[lab] : 0.f) - l;
  }
}

// Single block.  Sequence sums in fp64 (fixed order, deterministic), then the pair terms:
// z = beta((logp+ - ref+) - (logp- - ref-)), loss = softplus(-z), dloss_mean/dlogp+ = (sigmoid(z)-1) beta / n_pairs.
__global__ __launch_bounds__(256) void dpo_pairs_kernel(const float *__restrict__ logp_t, const int32_t *ft_seq_offsets,
                                                        const int32_t *prompt_lens, int n_seq, const float *ref_logp,
                                                        float beta, float *logp_out, float *loss_per_pair,
                                                        float *loss_mean, float *clpd, int32_t *win, float *dlogp) {
  __shared__ double part[256];
  __shared__ double seqsum[2];
  __shared__ double total;
  const int n_pairs = n_seq / 2;
  if (threadIdx.x == 0) total = 0.0;
  int base = 0;
  for (int pr = 0; pr < n_pairs; ++pr) {
    for (int q = 0; q < 2; ++q) {
      const int s = 2 * pr + q;
      const int n = (ft_seq_offsets[s + 1] - ft_seq_offsets[s]) - prompt_lens[s];
      double a = 0.0;
      for (int i = threadIdx.x; i < n; i += 256) a += (double)logp_t[base + i];
      part[threadIdx.x] = a;
      __syncthreads();
      for (int o = 128; o > 0; o >>= 1) {
        if (threadIdx.x < o) part[threadIdx.x] += part[threadIdx.x + o];
        __syncthreads();
      }
      if (threadIdx.x == 0) seqsum[q] = part[0];
      __syncthreads();
      base += n;
    }
    if (threadIdx.x == 0) {
      const double lp = seqsum[0], lm = seqsum[1];
      const double z = (double)beta * ((lp - (double)ref_logp[2 * pr]) - (lm - (double)ref_logp[2 * pr + 1]));
      const double loss = fmax(-z, 0.0) + log1p(exp(-fabs(z)));
      const double sig = 1.0 / (1.0 + exp(-z));
      const double c = (sig - 1.0) * (double)beta / (double)n_pairs;
      logp_out[2 * pr] = (float)lp;
      logp_out[2 * pr + 1] = (float)lm;
      loss_per_pair[pr] = (float)loss;
      if (clpd) clpd[pr] = (float)(lp - lm);
      if (win) win[pr] = (lp - lm) > 0.0 ? 1 : 0;
      dlogp[2 * pr] = (float)c;
      dlogp[2 * pr + 1] = (float)(-c);
      total += loss;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) *loss_mean = n_pairs > 0 ? (float)(total / (double)n_pairs) : 0.f;
}

__global__ __launch_bounds__(256) void dlogits_kernel(const float *__restrict__ logits, int V,
                                                      const int32_t *__restrict__ label,
                                                      const int32_t *__restrict__ seq_id, const float *__restrict__ lse,
                                                      const float *__restrict__ dlogp, bf16_t *__restrict__ dl) {
  const int r = blockIdx.x;
  const float c = dlogp[seq_id[r]], l = lse[r];
  const int lab = label[r];
  const float *row = logits + (size_t)r * V;
  bf16_t *out = dl + (size_t)r * V;
  for (int k = 4 * threadIdx.x; k < V; k += 1024) {
    const float4 v = *(const float4 *)(row + k);
    float o[4] = {-expf(v.x - l), -expf(v.y - l), -expf(v.z - l), -expf(v.w - l)};
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (k + j == lab) o[j] += 1.0f;
      o[j] *= c;
    }
    *(uint2 *)(out + k) = make_uint2(pack2(f2bf(o[0]), f2bf(o[1])), pack2(f2bf(o[2]), f2bf(o[3])));
  }
}

}  // namespace

hipError_t launch_loss_rows(const int32_t *ft_seq_offsets, const int32_t *prompt_lens, const int32_t *token_ids,
                            int n_seq, int32_t *row_idx, int32_t *label, int32_t *seq_id, hipStream_t st) {
  if (n_seq <= 0) return hipSuccess;
  hipLaunchKernelGGL(loss_rows_kernel, dim3(n_seq), dim3(256), 0, st, ft_seq_offsets, prompt_lens, token_ids, row_idx, label, seq_id);
  return hipGetLastError();
}

hipError_t launch_logsoftmax_gather(const float *logits, int rows, int V, const int32_t *label, float *logp_t,
                                    float *lse, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(logsoftmax_gather_kernel, dim3(rows), dim3(256), 0, st, logits, V, label, logp_t, lse);
  return hipGetLastError();
}

hipError_t launch_label_logit(const bf16_t *n_hi, const bf16_t *n_lo, const bf16_t *e, const int32_t *label, int rows, int d,
                              int V, float *logits, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(label_logit_kernel, dim3(cdiv(rows, 4)), dim3(256), 0, st, n_hi, n_lo, e, label, rows, d, V, logits);
  return hipGetLastError();
}

hipError_t launch_dpo_pairs(const float *logp_t, const int32_t *ft_seq_offsets, const int32_t *prompt_lens, int n_seq,
                            const float *ref_logp, float beta, float *logp_out, float *loss_per_pair, float *loss_mean,
                            float *clpd, int32_t *win, float *dlogp, hipStream_t st) {
  hipLaunchKernelGGL(dpo_pairs_kernel, dim3(1), dim3(256), 0, st, logp_t, ft_seq_offsets, prompt_lens, n_seq, ref_logp, beta, logp_out, loss_per_pair, loss_mean, clpd, win, dlogp);
  return hipGetLastError();
}

hipError_t launch_loss_rows_shared(const int32_t *pair_offsets, const int32_t *prompt_lens, const int32_t *chosen_lens,
                                   const int32_t *token_ids, int n_pairs, int32_t *row_idx, int32_t *label, int32_t *seq_id,
                                   int32_t *partner, int32_t *vseq_off, int32_t *vprompt, hipStream_t st) {
  if (n_pairs <= 0) return hipSuccess;
  hipLaunchKernelGGL(loss_rows_shared_kernel, dim3(n_pairs), dim3(256), 0, st, pair_offsets, prompt_lens, chosen_lens, token_ids, n_pairs,
                     row_idx, label, seq_id, partner, vseq_off, vprompt);
  return hipGetLastError();
}

hipError_t launch_scatter_rows(const float *src, const int32_t *row_idx, const int32_t *partner, int rows, int d, float *dst,
                               hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(scatter_rows_kernel, dim3(rows), dim3(256), 0, st, src, row_idx, partner, d, dst);
  return hipGetLastError();
}

hipError_t launch_dlogits(const float *logits, int rows, int V, const int32_t *label, const int32_t *seq_id,
                          const float *lse, const float *dlogp, bf16_t *dl, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(dlogits_kernel, dim3(rows), dim3(256), 0, st, logits, V, label, seq_id, lse, dlogp, dl);
  return hipGetLastError();
}
