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

// One block of 1024 threads per loss row.  The V logits of the row are read once into registers
// (NCH float4 per thread), reduced to (max, sum) and, when dl is wanted, turned into
//   dl[r, j] = [j == label[r]] - exp(logits[r, j] - lse[r])        (bf16)
// i.e. d log p(label) / d logits, WITHOUT the factor dL/dlog p of the row's sequence: that factor
// depends on the pair loss, which is known only after every row of the pair is done; it is applied
// to the (much smaller) products of dl afterwards (scale_rows_kernel).  NCH == 0: rows longer than
// the register budget are read twice.
template <int NCH>
__global__ __launch_bounds__(1024) void logsoftmax_dl_kernel(const float *__restrict__ logits, int V,
                                                             const int32_t *__restrict__ label, float *__restrict__ logp_t,
                                                             float *__restrict__ lse, bf16_t *__restrict__ dl) {
  __shared__ float red[16];
  const int r = blockIdx.x;
  const float *row = logits + (size_t)r * V;
  const int lab = label[r];
  float4 v[NCH > 0 ? NCH : 1];
  float m = -INFINITY, s = 0.f;
  if constexpr (NCH > 0) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int k = 4 * (threadIdx.x + 1024 * i);             // V % 4 == 0
      v[i] = k < V ? *(const float4 *)(row + k) : make_float4(-INFINITY, -INFINITY, -INFINITY, -INFINITY);
      m = fmaxf(m, fmaxf(fmaxf(v[i].x, v[i].y), fmaxf(v[i].z, v[i].w)));
    }
    if (m > -INFINITY) {
#pragma unroll
      for (int i = 0; i < NCH; ++i) s += expf(v[i].x - m) + expf(v[i].y - m) + expf(v[i].z - m) + expf(v[i].w - m);
    }
  } else {
    for (int k = 4 * threadIdx.x; k < V; k += 4096) {
      const float4 w = *(const float4 *)(row + k);
      const float mx = fmaxf(fmaxf(w.x, w.y), fmaxf(w.z, w.w));
      if (mx > m) { s *= expf(m - mx); m = mx; }
      s += expf(w.x - m) + expf(w.y - m) + expf(w.z - m) + expf(w.w - m);
    }
  }
  const float mb = block_max<1024>(m, red);
  s = (m == -INFINITY) ? 0.f : s * expf(m - mb);
  const float sb = block_sum<1024>(s, red);
  const float l = mb + logf(sb);
  if (threadIdx.x == 0) {
    lse[r] = l;
    logp_t[r] = (lab >= 0 && lab < V ? row[lab] : 0.f) - l;
  }
  if (!dl) return;
  bf16_t *out = dl + (size_t)r * V;
  auto emit = [&](int k, const float4 &w) {
    float o[4] = {-expf(w.x - l), -expf(w.y - l), -expf(w.z - l), -expf(w.w - l)};
#pragma unroll
    for (int j = 0; j < 4; ++j)
      if (k + j == lab) o[j] += 1.0f;
    *(uint2 *)(out + k) = make_uint2(cvt_pk_bf16(o[0], o[1]), cvt_pk_bf16(o[2], o[3]));
  };
  if constexpr (NCH > 0) {
#pragma unroll
    for (int i = 0; i < NCH; ++i) {
      const int k = 4 * (threadIdx.x + 1024 * i);
      if (k < V) emit(k, v[i]);
    }
  } else {
    for (int k = 4 * threadIdx.x; k < V; k += 4096) emit(k, *(const float4 *)(row + k));
  }
}

// First-order correction of log p(label) for the rounding of the normalised rows to bf16 in a ONE-PASS
// head.  With n = n_hi + n_lo and logits formed from n_hi alone, every logit of the row is short of
// n_lo . E_j; to first order
//   log p(label) - log p(label)|n_hi  =  n_lo . E_label - sum_j p_j (n_lo . E_j)  =  n_lo . u,
//   u = E_label - sum_j p_j E_j = dl[r, :] E
// and u is the product the backward pass forms anyway (the gradient with respect to the normalised
// row, before its sequence factor).  What is left is second order in n_lo (about 1e-7 per row) and
// nearly the same for the two sequences of a pair.  One wave per loss row.
__global__ __launch_bounds__(256) void logp_correct_kernel(const bf16_t *__restrict__ n_lo, const float *__restrict__ u, int rows, int d,
                                                           float *__restrict__ logp_t) {
  const int lane = threadIdx.x & 63, r = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (r >= rows) return;
  const bf16_t *a = n_lo + (size_t)r * d;
  const float *b = u + (size_t)r * d;
  float s = 0.f;
  for (int k = lane * 4; k < d; k += 256) {        // d % 4 == 0
    const uint2 ua = *(const uint2 *)(a + k);
    const float4 ub = *(const float4 *)(b + k);
    s += __uint_as_float(ua.x << 16) * ub.x + __uint_as_float(ua.x & 0xffff0000u) * ub.y +
         __uint_as_float(ua.y << 16) * ub.z + __uint_as_float(ua.y & 0xffff0000u) * ub.w;
  }
  s = wave_sum(s);
  if (lane == 0) logp_t[r] += s;
}

// After the pair losses: row r belongs to sequence seq_id[r], whose dL/dlog p is c = dlogp[seq_id[r]].
//   dn[r, :] = c * u[r, :]  (in place, fp32; skipped when u is null)
//   n_c[r, :] = bf16(c * n_hi[r, :])  (skipped when n_c is null), so that dE = dl^T n_c.
__global__ __launch_bounds__(256) void scale_rows_kernel(float *__restrict__ u, const bf16_t *__restrict__ n_hi, bf16_t *__restrict__ n_c,
                                                         const int32_t *__restrict__ seq_id, const float *__restrict__ dlogp, int d) {
  const int r = blockIdx.x;
  const float c = dlogp[seq_id[r]];
  for (int k = 4 * threadIdx.x; k < d; k += 1024) {        // d % 4 == 0
    if (u) {
      float4 w = *(float4 *)(u + (size_t)r * d + k);
      w.x *= c; w.y *= c; w.z *= c; w.w *= c;
      *(float4 *)(u + (size_t)r * d + k) = w;
    }
    if (n_c) {
      const uint2 a = *(const uint2 *)(n_hi + (size_t)r * d + k);
      *(uint2 *)(n_c + (size_t)r * d + k) = make_uint2(cvt_pk_bf16(c * __uint_as_float(a.x << 16), c * __uint_as_float(a.x & 0xffff0000u)),
                                                       cvt_pk_bf16(c * __uint_as_float(a.y << 16), c * __uint_as_float(a.y & 0xffff0000u)));
    }
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

}  // namespace

hipError_t launch_loss_rows(const int32_t *ft_seq_offsets, const int32_t *prompt_lens, const int32_t *token_ids,
                            int n_seq, int32_t *row_idx, int32_t *label, int32_t *seq_id, hipStream_t st) {
  if (n_seq <= 0) return hipSuccess;
  hipLaunchKernelGGL(loss_rows_kernel, dim3(n_seq), dim3(256), 0, st, ft_seq_offsets, prompt_lens, token_ids, row_idx, label, seq_id);
  return hipGetLastError();
}

hipError_t launch_logsoftmax_dl(const float *logits, int rows, int V, const int32_t *label, float *logp_t, float *lse, bf16_t *dl,
                               hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  if (V % 4) return hipErrorInvalidValue;
  if (V <= 4096 * 8) hipLaunchKernelGGL(logsoftmax_dl_kernel<8>, dim3(rows), dim3(1024), 0, st, logits, V, label, logp_t, lse, dl);
  else if (V <= 4096 * 16) hipLaunchKernelGGL(logsoftmax_dl_kernel<16>, dim3(rows), dim3(1024), 0, st, logits, V, label, logp_t, lse, dl);
  else hipLaunchKernelGGL(logsoftmax_dl_kernel<0>, dim3(rows), dim3(1024), 0, st, logits, V, label, logp_t, lse, dl);
  return hipGetLastError();
}

hipError_t launch_logp_correct(const bf16_t *n_lo, const float *u, int rows, int d, float *logp_t, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(logp_correct_kernel, dim3(cdiv(rows, 4)), dim3(256), 0, st, n_lo, u, rows, d, logp_t);
  return hipGetLastError();
}

hipError_t launch_scale_rows(float *u, const bf16_t *n_hi, bf16_t *n_c, const int32_t *seq_id, const float *dlogp, int rows, int d,
                             hipStream_t st) {
  if (rows <= 0 || (!u && !n_c)) return hipSuccess;
  hipLaunchKernelGGL(scale_rows_kernel, dim3(rows), dim3(256), 0, st, u, n_hi, n_c, seq_id, dlogp, d);
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
