// HBM-bound row kernels: RMSNorm, rotary embedding, SwiGLU, operand splitting (fwd and bwd).
#include "kernels.h"

namespace {

template <bool BF16>
__device__ __forceinline__ void ld4(const void *p, size_t i, float v[4]) {
  if constexpr (BF16) {
    const uint2 u = *(const uint2 *)((const bf16_t *)p + i);
    v[0] = __uint_as_float(u.x << 16); v[1] = __uint_as_float(u.x & 0xffff0000u);
    v[2] = __uint_as_float(u.y << 16); v[3] = __uint_as_float(u.y & 0xffff0000u);
  } else {
    const float4 f = *(const float4 *)((const float *)p + i);
    v[0] = f.x; v[1] = f.y; v[2] = f.z; v[3] = f.w;
  }
}

__device__ __forceinline__ void st4_split(bf16_t *hi, bf16_t *lo, size_t i, const float v[4]) {
  bf16_t h[4], l[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) split_bf(v[j], h[j], l[j]);
  *(uint2 *)(hi + i) = make_uint2(pack2(h[0], h[1]), pack2(h[2], h[3]));
  if (lo) *(uint2 *)(lo + i) = make_uint2(pack2(l[0], l[1]), pack2(l[2], l[3]));
}

// ------------------------------------------------------------------ RMSNorm forward
template <bool XBF, bool GBF>
__global__ __launch_bounds__(256) void rmsnorm_fwd_kernel(const void *x, const int32_t *row_idx, const void *g, int d,
                                                          float eps, bf16_t *hi, bf16_t *lo, float *rstd) {
  __shared__ float red[4];
  const int r = blockIdx.x;
  const size_t xin = (size_t)(row_idx ? row_idx[r] : r) * d, xo = (size_t)r * d;
  float ss = 0.f;
  for (int k = 4 * threadIdx.x; k < d; k += 1024) {
    float v[4];
    ld4<XBF>(x, xin + k, v);
    ss += v[0] * v[0] + v[1] * v[1] + v[2] * v[2] + v[3] * v[3];
  }
  ss = block_sum<256>(ss, red);
  const float rs = 1.0f / sqrtf(ss / (float)d + eps);
  if (rstd && threadIdx.x == 0) rstd[r] = rs;
  for (int k = 4 * threadIdx.x; k < d; k += 1024) {
    float v[4], gg[4];
    ld4<XBF>(x, xin + k, v);
    ld4<GBF>(g, k, gg);
#pragma unroll
    for (int j = 0; j < 4; ++j) v[j] = v[j] * rs * gg[j];
    st4_split(hi, lo, xo + k, v);
  }
}

// ------------------------------------------------------------------ RMSNorm backward
constexpr int RB_MAXV = 8;   // d <= 8192
// One block per partial row of dg; a block walks rows r = blockIdx.x, + gridDim.x, ...  NV = float4
// chunks per thread (d <= 1024 NV): the row of dy and of x stays in registers between the reduction
// and the output pass, and g is read once per block.
template <bool XBF, bool GBF, int NV>
__global__ __launch_bounds__(256) void rmsnorm_bwd_kernel(const float *dy, const void *x, const int32_t *row_idx,
                                                          const void *g, const float *rstd, const float *resid,
                                                          int rows, int d, float *dx_out, bf16_t *dx_bf,
                                                          float *dg_partial, int dense_out) {
  __shared__ float red[4];
  float dgacc[NV][4], gg[NV][4];
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int k = 4 * threadIdx.x + 1024 * i;
#pragma unroll
    for (int j = 0; j < 4; ++j) dgacc[i][j] = gg[i][j] = 0.f;
    if (k < d) ld4<GBF>(g, k, gg[i]);
  }
  for (int r = blockIdx.x; r < rows; r += gridDim.x) {
    const size_t xr = (size_t)(row_idx ? row_idx[r] : r) * d, yr = (size_t)r * d;
    float dv[NV][4], xv[NV][4], rr[NV][4];
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int k = 4 * threadIdx.x + 1024 * i;
#pragma unroll
      for (int j = 0; j < 4; ++j) dv[i][j] = xv[i][j] = rr[i][j] = 0.f;
      if (k < d) {
        ld4<false>(dy, yr + k, dv[i]);
        ld4<XBF>(x, xr + k, xv[i]);
        if (resid) ld4<false>(resid, yr + k, rr[i]);
      }
    }
    const float rs = rstd[r];
    float s = 0.f;
#pragma unroll
    for (int i = 0; i < NV; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        s += dv[i][j] * gg[i][j] * xv[i][j];
        dgacc[i][j] += dv[i][j] * xv[i][j] * rs;
      }
    s = block_sum<256>(s, red);
    const float c = rs * rs * rs * s / (float)d;
    const size_t orow = dense_out ? yr : xr;      // dense: output row r (may be dy itself), else the gathered row
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int k = 4 * threadIdx.x + 1024 * i;
      if (k < d) {
        float o[4];
#pragma unroll
        for (int j = 0; j < 4; ++j) o[j] = rr[i][j] + rs * dv[i][j] * gg[i][j] - xv[i][j] * c;
        *(float4 *)(dx_out + orow + k) = make_float4(o[0], o[1], o[2], o[3]);
        if (dx_bf) *(uint2 *)(dx_bf + orow + k) = make_uint2(pack2(f2bf(o[0]), f2bf(o[1])), pack2(f2bf(o[2]), f2bf(o[3])));
      }
    }
  }
#pragma unroll
  for (int i = 0; i < NV; ++i) {
    const int k = 4 * threadIdx.x + 1024 * i;
    if (k < d) *(float4 *)(dg_partial + (size_t)blockIdx.x * d + k) = make_float4(dgacc[i][0], dgacc[i][1], dgacc[i][2], dgacc[i][3]);
  }
}

// Column sums of the partial rows in two launches: slice y of COLSUM_SLICES sums the rows y, y + S,
// y + 2S, ... of 256 adjacent columns (1 KB contiguous per row, eight loads in flight per thread) into
// row y of a scratch buffer; the second launch (n_slices rows, slices == 1) adds those rows in a fixed
// order: deterministic.  (A block that walks many rows of a narrow column strip puts all its loads, a
// power-of-two stride apart, on the same memory channel.)
__global__ __launch_bounds__(256) void colsum_kernel(const float *part, int n_part, int d, int slices, float *out, int accumulate) {
  const int j = blockIdx.x * 256 + threadIdx.x, y = blockIdx.y;
  if (j >= d) return;
  float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
  int i = y;
  for (; i + 7 * slices < n_part; i += 8 * slices) {
#pragma unroll
    for (int u = 0; u < 8; ++u) a[u] += part[(size_t)(i + slices * u) * d + j];
  }
  for (; i < n_part; i += slices) a[0] += part[(size_t)i * d + j];
  const float t = ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]));
  float *o = out + (size_t)y * d + j;
  *o = accumulate ? *o + t : t;
}

// ------------------------------------------------------------------ rotary embedding
// cs[i] = (cos, sin) of pos * inv_freq[i]; the angle is formed and reduced in fp64.
__device__ __forceinline__ void rope_table(float2 *cs, int pos, const double *inv_freq, int half) {
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    double s, c;
    sincos((double)pos * inv_freq[i], &s, &c);
    cs[i] = make_float2((float)c, (float)s);
  }
  __syncthreads();
}

template <bool CBF>
__global__ __launch_bounds__(256) void rope_split_kernel(const float *qkv, const int32_t *positions,
                                                         const double *inv_freq, int Hq, int Hkv, int hd, bf16_t *q_hi,
                                                         bf16_t *k_hi, bf16_t *v_hi, bf16_t *q_lo, bf16_t *k_lo,
                                                         bf16_t *v_lo, const int32_t *slot_mapping, void *cache_k,
                                                         void *cache_v, long long num_slots, int block_size) {
  __shared__ float2 cs[64];
  const int r = blockIdx.x, half = hd >> 1;
  rope_table(cs, positions[r], inv_freq, half);
  const int qd = Hq * hd, kd = Hkv * hd, nq = qd + 2 * kd;
  const float *in = qkv + (size_t)r * nq;
  long long slot = -1;
  if (slot_mapping) {
    slot = slot_mapping[r];
    if (slot >= num_slots) slot = -1;
  }
  const long long cbase = slot >= 0 ? (slot / block_size) * (long long)Hkv * block_size * hd + (slot % block_size) * (long long)hd : 0;
  const int npair = (Hq + Hkv) * half;
  for (int idx = threadIdx.x; idx < npair; idx += 256) {
    const int head = idx / half, i = idx - head * half;
    const float a = in[head * hd + i], b = in[head * hd + i + half];
    const float2 t = cs[i];
    const float ra = a * t.x - b * t.y, rb = b * t.x + a * t.y;
    bf16_t ha, la, hb, lb;
    split_bf(ra, ha, la);
    split_bf(rb, hb, lb);
    if (head < Hq) {
      const size_t o = (size_t)r * qd + head * hd + i;
      q_hi[o] = ha; q_hi[o + half] = hb;
      if (q_lo) { q_lo[o] = la; q_lo[o + half] = lb; }
    } else {
      const int kh = head - Hq;
      const size_t o = (size_t)r * kd + kh * hd + i;
      k_hi[o] = ha; k_hi[o + half] = hb;
      if (k_lo) { k_lo[o] = la; k_lo[o + half] = lb; }
      if (slot >= 0) {
        const long long c = cbase + (long long)kh * block_size * hd + i;
        if constexpr (CBF) { ((bf16_t *)cache_k)[c] = ha; ((bf16_t *)cache_k)[c + half] = hb; }
        else { ((float *)cache_k)[c] = ra; ((float *)cache_k)[c + half] = rb; }
      }
    }
  }
  for (int idx = threadIdx.x; idx < kd; idx += 256) {
    const float v = in[qd + kd + idx];
    bf16_t h, l;
    split_bf(v, h, l);
    v_hi[(size_t)r * kd + idx] = h;
    if (v_lo) v_lo[(size_t)r * kd + idx] = l;
    if (slot >= 0) {
      const int kh = idx / hd, e = idx - kh * hd;
      const long long c = cbase + (long long)kh * block_size * hd + e;
      if constexpr (CBF) ((bf16_t *)cache_v)[c] = h;
      else ((float *)cache_v)[c] = v;
    }
  }
}

__global__ __launch_bounds__(64) void rope_table_kernel(const int32_t *__restrict__ positions, const double *__restrict__ inv_freq,
                                                        int half, float2 *__restrict__ cs) {
  const int r = blockIdx.x, i = threadIdx.x;
  if (i >= half) return;
  double sn, c;
  sincos((double)positions[r] * inv_freq[i], &sn, &c);
  cs[(size_t)r * half + i] = make_float2((float)c, (float)sn);
}

// ------------------------------------------------------------------ SwiGLU
// 8 hidden units per thread (16-byte accesses); F % 8 == 0.
__global__ __launch_bounds__(256) void swiglu_bwd_kernel(const bf16_t *__restrict__ dhm, const bf16_t *__restrict__ gu, int F,
                                                         bf16_t *__restrict__ dgu) {
  const int r = blockIdx.x;
  const int k = 8 * (blockIdx.y * 256 + threadIdx.x);
  if (k >= F) return;
  const uint4 gq = *(const uint4 *)(gu + (size_t)r * 2 * F + k), uq = *(const uint4 *)(gu + (size_t)r * 2 * F + F + k);
  const uint4 dq = *(const uint4 *)(dhm + (size_t)r * F + k);
  const uint32_t gw[4] = {gq.x, gq.y, gq.z, gq.w}, uw[4] = {uq.x, uq.y, uq.z, uq.w}, dw[4] = {dq.x, dq.y, dq.z, dq.w};
  uint32_t og[4], ou[4];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    float dg[2], du[2];
#pragma unroll
    for (int e = 0; e < 2; ++e) {
      const float g = e ? __uint_as_float(gw[j] & 0xffff0000u) : __uint_as_float(gw[j] << 16);
      const float u = e ? __uint_as_float(uw[j] & 0xffff0000u) : __uint_as_float(uw[j] << 16);
      const float dh = e ? __uint_as_float(dw[j] & 0xffff0000u) : __uint_as_float(dw[j] << 16);
      const float sg = 1.0f / (1.0f + expf(-g));
      du[e] = dh * g * sg;
      dg[e] = dh * u * sg * (1.0f + g * (1.0f - sg));
    }
    og[j] = cvt_pk_bf16(dg[0], dg[1]);
    ou[j] = cvt_pk_bf16(du[0], du[1]);
  }
  *(uint4 *)(dgu + (size_t)r * 2 * F + k) = make_uint4(og[0], og[1], og[2], og[3]);
  *(uint4 *)(dgu + (size_t)r * 2 * F + F + k) = make_uint4(ou[0], ou[1], ou[2], ou[3]);
}

__global__ __launch_bounds__(256) void split_f32_kernel(const float *src, size_t n, bf16_t *hi, bf16_t *lo) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
    bf16_t h, l;
    split_bf(src[i], h, l);
    hi[i] = h;
    if (lo) lo[i] = l;
  }
}

__global__ __launch_bounds__(256) void sum_partials_kernel(const float *part, int n_part, size_t n, float *out) {
  const size_t stride = (size_t)gridDim.x * 256 * 4;
  for (size_t i = ((size_t)blockIdx.x * 256 + threadIdx.x) * 4; i < n; i += stride) {   // n % 4 == 0
    float4 a = *(const float4 *)(part + i);
    for (int s = 1; s < n_part; ++s) {
      const float4 b = *(const float4 *)(part + (size_t)s * n + i);
      a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
    }
    *(float4 *)(out + i) = a;
  }
}

__global__ __launch_bounds__(256) void fill_f32_kernel(float *dst, size_t n, float v) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) dst[i] = v;
}

}  // namespace

hipError_t launch_rmsnorm_fwd(const void *x, bool x_bf16, const int32_t *row_idx, const void *g, bool g_bf16, int rows,
                              int d, float eps, bf16_t *hi, bf16_t *lo, float *rstd, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  dim3 grid(rows), blk(256);
  if (x_bf16 && g_bf16) hipLaunchKernelGGL((rmsnorm_fwd_kernel<true, true>), grid, blk, 0, st, x, row_idx, g, d, eps, hi, lo, rstd);
  else if (!x_bf16 && g_bf16) hipLaunchKernelGGL((rmsnorm_fwd_kernel<false, true>), grid, blk, 0, st, x, row_idx, g, d, eps, hi, lo, rstd);
  else if (!x_bf16 && !g_bf16) hipLaunchKernelGGL((rmsnorm_fwd_kernel<false, false>), grid, blk, 0, st, x, row_idx, g, d, eps, hi, lo, rstd);
  else hipLaunchKernelGGL((rmsnorm_fwd_kernel<true, false>), grid, blk, 0, st, x, row_idx, g, d, eps, hi, lo, rstd);
  return hipGetLastError();
}

template <bool XBF, bool GBF>
static void rmsnorm_bwd_nv(int nv, dim3 grid, hipStream_t st, const float *dy, const void *x, const int32_t *row_idx, const void *g,
                           const float *rstd, const float *resid, int rows, int d, float *dx_out, bf16_t *dx_bf,
                           float *dg_partial, int dense_out) {
  const dim3 blk(256);
  if (nv <= 1) hipLaunchKernelGGL((rmsnorm_bwd_kernel<XBF, GBF, 1>), grid, blk, 0, st, dy, x, row_idx, g, rstd, resid, rows, d, dx_out, dx_bf, dg_partial, dense_out);
  else if (nv <= 2) hipLaunchKernelGGL((rmsnorm_bwd_kernel<XBF, GBF, 2>), grid, blk, 0, st, dy, x, row_idx, g, rstd, resid, rows, d, dx_out, dx_bf, dg_partial, dense_out);
  else if (nv <= 4) hipLaunchKernelGGL((rmsnorm_bwd_kernel<XBF, GBF, 4>), grid, blk, 0, st, dy, x, row_idx, g, rstd, resid, rows, d, dx_out, dx_bf, dg_partial, dense_out);
  else hipLaunchKernelGGL((rmsnorm_bwd_kernel<XBF, GBF, RB_MAXV>), grid, blk, 0, st, dy, x, row_idx, g, rstd, resid, rows, d, dx_out, dx_bf, dg_partial, dense_out);
}

hipError_t launch_rmsnorm_bwd(const float *dy, const void *x, bool x_bf16, const int32_t *row_idx, const void *g,
                              bool g_bf16, const float *rstd, const float *resid, int rows, int d, float *dx_out,
                              bf16_t *dx_bf, float *dg_partial, int n_part, hipStream_t st, int dense_out) {
  if (rows <= 0 || n_part <= 0) return hipSuccess;
  if (d > 1024 * RB_MAXV) return hipErrorInvalidValue;
  const dim3 grid(n_part);
  const int nv = (d + 1023) / 1024;
  if (x_bf16 && g_bf16) rmsnorm_bwd_nv<true, true>(nv, grid, st, dy, x, row_idx, g, rstd, resid, rows, d, dx_out, dx_bf, dg_partial, dense_out);
  else if (!x_bf16 && g_bf16) rmsnorm_bwd_nv<false, true>(nv, grid, st, dy, x, row_idx, g, rstd, resid, rows, d, dx_out, dx_bf, dg_partial, dense_out);
  else if (!x_bf16 && !g_bf16) rmsnorm_bwd_nv<false, false>(nv, grid, st, dy, x, row_idx, g, rstd, resid, rows, d, dx_out, dx_bf, dg_partial, dense_out);
  else rmsnorm_bwd_nv<true, false>(nv, grid, st, dy, x, row_idx, g, rstd, resid, rows, d, dx_out, dx_bf, dg_partial, dense_out);
  return hipGetLastError();
}

hipError_t launch_colsum(const float *part, int n_part, int d, float *scratch, float *out, int accumulate, hipStream_t st) {
  const int slices = n_part >= 4 * COLSUM_SLICES ? COLSUM_SLICES : 1;
  const dim3 blk(256);
  if (slices > 1) {
    hipLaunchKernelGGL(colsum_kernel, dim3(cdiv(d, 256), slices), blk, 0, st, part, n_part, d, slices, scratch, 0);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    part = scratch;
    n_part = slices;
  }
  hipLaunchKernelGGL(colsum_kernel, dim3(cdiv(d, 256), 1), blk, 0, st, part, n_part, d, 1, out, accumulate);
  return hipGetLastError();
}

hipError_t launch_rope_split(const float *qkv, const int32_t *positions, const double *inv_freq, int rows, int Hq,
                             int Hkv, int hd, bf16_t *q_hi, bf16_t *k_hi, bf16_t *v_hi, bf16_t *q_lo, bf16_t *k_lo,
                             bf16_t *v_lo, const int32_t *slot_mapping, void *cache_k, void *cache_v, bool cache_bf16,
                             long long num_slots, int block_size, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  if (hd > 128) return hipErrorInvalidValue;
  if (cache_bf16)
    hipLaunchKernelGGL((rope_split_kernel<true>), dim3(rows), dim3(256), 0, st, qkv, positions, inv_freq, Hq, Hkv, hd, q_hi, k_hi, v_hi, q_lo, k_lo, v_lo, slot_mapping, cache_k, cache_v, num_slots, block_size);
  else
    hipLaunchKernelGGL((rope_split_kernel<false>), dim3(rows), dim3(256), 0, st, qkv, positions, inv_freq, Hq, Hkv, hd, q_hi, k_hi, v_hi, q_lo, k_lo, v_lo, slot_mapping, cache_k, cache_v, num_slots, block_size);
  return hipGetLastError();
}

hipError_t launch_rope_table(const int32_t *positions, const double *inv_freq, int rows, int hd, float2 *cs, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  if (hd > 128) return hipErrorInvalidValue;
  hipLaunchKernelGGL(rope_table_kernel, dim3(rows), dim3(64), 0, st, positions, inv_freq, hd >> 1, cs);
  return hipGetLastError();
}

hipError_t launch_swiglu_bwd(const bf16_t *dhm, const bf16_t *gu, int rows, int F, bf16_t *dgu, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  if (F % 8) return hipErrorInvalidValue;
  hipLaunchKernelGGL(swiglu_bwd_kernel, dim3(rows, cdiv(F, 2048)), dim3(256), 0, st, dhm, gu, F, dgu);
  return hipGetLastError();
}

hipError_t launch_split_f32(const float *src, size_t n, bf16_t *hi, bf16_t *lo, hipStream_t st) {
  if (n == 0) return hipSuccess;
  const unsigned blocks = (unsigned)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  hipLaunchKernelGGL(split_f32_kernel, dim3(blocks), dim3(256), 0, st, src, n, hi, lo);
  return hipGetLastError();
}

namespace {
__global__ __launch_bounds__(256) void head_norm_stats_kernel(const float *__restrict__ norms, const int32_t *__restrict__ t_count,
                                                              int n, int H, float *__restrict__ abar, int32_t *__restrict__ last_used,
                                                              int window, float tau, int32_t *__restrict__ prune) {
  const int i = blockIdx.x * 256 + threadIdx.x;
  if (i >= n * H) return;
  const int t = t_count[i / H];
  if (t < 1) return;              // a request that has had no decode iteration: nothing to average over
  const float v = norms[i], a = abar[i];
  abar[i] = a + (v - a) / (float)t;
  if (prune) {
    const bool low = v < tau;
    prune[i] = (t - last_used[i] > window || low) ? 1 : 0;
    if (!low) last_used[i] = t;
  }
}
}  // namespace

hipError_t launch_head_norm_stats(const float *norms, const int32_t *t_count, int n, int H, float *abar, int32_t *last_used,
                                  int window, float tau, int32_t *prune, hipStream_t st) {
  if (n <= 0 || H <= 0) return hipSuccess;
  hipLaunchKernelGGL(head_norm_stats_kernel, dim3((unsigned)cdiv(n * H, 256)), dim3(256), 0, st, norms, t_count, n, H, abar, last_used, window, tau, prune);
  return hipGetLastError();
}

hipError_t launch_fill_f32(float *dst, size_t n, float v, hipStream_t st) {
  if (n == 0) return hipSuccess;
  const unsigned blocks = (unsigned)((n + 255) / 256 < 4096 ? (n + 255) / 256 : 4096);
  hipLaunchKernelGGL(fill_f32_kernel, dim3(blocks), dim3(256), 0, st, dst, n, v);
  return hipGetLastError();
}

hipError_t launch_sum_partials(const float *part, int n_part, size_t n, float *out, hipStream_t st) {
  if (n == 0) return hipSuccess;
  if (n % 4) return hipErrorInvalidValue;
  const size_t want = (n / 4 + 255) / 256;
  hipLaunchKernelGGL(sum_partials_kernel, dim3((unsigned)(want < 4096 ? want : 4096)), dim3(256), 0, st, part, n_part, n, out);
  return hipGetLastError();
}
