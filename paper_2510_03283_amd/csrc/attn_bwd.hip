// Backward of the varlen causal attention of the fine-tune sequences (bf16 MFMA, fp32 outputs).
//
// Two kernels, each free of atomics and of cross-lane transposes:
//  * dq kernel:  a wave owns 32 queries (a lane owns one query column of S^T = K Q^T and of
//    dP^T = V dO^T), walks the keys, and accumulates dQ^T = K^T dS^T.
//  * dkdv kernel: a wave owns 32 keys (a lane owns one key column of S = Q K^T and dP = dO V^T),
//    walks the queries of every query head of its GQA group, and accumulates
//    dV^T = dO^T P and dK^T = Q^T dS.
// P is recomputed from the saved log-sum-exp; D = rowsum(dO * O) comes from a small pre-kernel.
// Tiles that feed the "transposed" products are transposed while they are staged into LDS, with
// bits 2 and 3 of the row index swapped so that a lane's 8 reduction indices are contiguous.
#include "kernels.h"

namespace {

constexpr int TB = 64;    // rows per staged LDS tile

__device__ __forceinline__ bf16x8_t as_bf8(uint4 u) { return __builtin_bit_cast(bf16x8_t, u); }

// dst[TB][HD+8] <- rows row0 .. row0+TB-1 of src (pitch ld), zero beyond row_end.
template <int HD>
__device__ __forceinline__ void stage_rows(bf16_t *dst, const bf16_t *src, size_t ld, int row0, int row_end) {
  for (int c = threadIdx.x; c < TB * HD / 8; c += 256) {
    const int row = c / (HD / 8), ch = c % (HD / 8);
    uint4 v = make_uint4(0, 0, 0, 0);
    if (row0 + row < row_end) v = *(const uint4 *)(src + (size_t)(row0 + row) * ld + ch * 8);
    *(uint4 *)(dst + row * (HD + 8) + ch * 8) = v;
  }
}

// dst[HD][TB+8] <- transpose of the same rows; source row i lands in column swap23(i).
template <int HD>
__device__ __forceinline__ void stage_rows_t(bf16_t *dst, const bf16_t *src, size_t ld, int row0, int row_end) {
  for (int c = threadIdx.x; c < (TB / 4) * (HD / 8); c += 256) {
    const int hb = c % (HD / 8), rq = c / (HD / 8);
    uint32_t d[4][4];
#pragma unroll
    for (int jj = 0; jj < 4; ++jj) {
      uint4 v = make_uint4(0, 0, 0, 0);
      const int row = row0 + 4 * rq + jj;
      if (row < row_end) v = *(const uint4 *)(src + (size_t)row * ld + hb * 8);
      d[jj][0] = v.x; d[jj][1] = v.y; d[jj][2] = v.z; d[jj][3] = v.w;
    }
    const int rq2 = (rq & ~3) | ((rq & 1) << 1) | ((rq >> 1) & 1);
#pragma unroll
    for (int m = 0; m < 8; ++m) {
      uint32_t w0, w1;
      if (m & 1) {
        w0 = (d[0][m >> 1] >> 16) | (d[1][m >> 1] & 0xffff0000u);
        w1 = (d[2][m >> 1] >> 16) | (d[3][m >> 1] & 0xffff0000u);
      } else {
        w0 = (d[0][m >> 1] & 0xffffu) | (d[1][m >> 1] << 16);
        w1 = (d[2][m >> 1] & 0xffffu) | (d[3][m >> 1] << 16);
      }
      *(uint2 *)(dst + (hb * 8 + m) * (TB + 8) + 4 * rq2) = make_uint2(w0, w1);
    }
  }
}

__device__ __forceinline__ bf16x8_t pack8(const float *v) {
  return as_bf8(make_uint4(pack2(f2bf(v[0]), f2bf(v[1])), pack2(f2bf(v[2]), f2bf(v[3])),
                           pack2(f2bf(v[4]), f2bf(v[5])), pack2(f2bf(v[6]), f2bf(v[7]))));
}

// ------------------------------------------------------------------ D = rowsum(dO * O)
__global__ __launch_bounds__(256) void attn_dvec_kernel(const bf16_t *__restrict__ o, const bf16_t *__restrict__ d_o,
                                                        int Hq, int hd, float *__restrict__ dvec) {
  const int r = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  for (int h = wave; h < Hq; h += 4) {
    const size_t b = ((size_t)r * Hq + h) * hd;
    float s = 0.f;
    for (int e = lane; e < hd; e += 64) s += bf2f(o[b + e]) * bf2f(d_o[b + e]);
    s = wave_sum(s);
    if (lane == 0) dvec[(size_t)r * Hq + h] = s;
  }
}

// ------------------------------------------------------------------ dQ
template <int HD>
__global__ __launch_bounds__(256) void attn_bwd_dq_kernel(const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
                                                          const bf16_t *__restrict__ v, const bf16_t *__restrict__ d_o,
                                                          const float *__restrict__ lse, const float *__restrict__ dvec,
                                                          const int32_t *__restrict__ seg, int row_base, int Hq, int Hkv,
                                                          float *__restrict__ dq) {
  constexpr int KP = HD + 8, TP = TB + 8, NKK = HD / 16, NOT = HD / 32;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t *Ks = (bf16_t *)smem_raw;          // [TB][KP]
  bf16_t *Vs = Ks + TB * KP;                // [TB][KP]
  bf16_t *Kt = Vs + TB * KP;                // [HD][TP]
  const int s = blockIdx.y, h = blockIdx.z, kvh = h / (Hq / Hkv);
  const int r0 = seg[s] - row_base, L = seg[s + 1] - seg[s];
  const int q0 = (gridDim.x - 1 - blockIdx.x) * 128;
  if (q0 >= L) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, j = lane & 31;
  const int qw0 = q0 + wave * 32, qi = qw0 + j;
  const size_t qld = (size_t)Hq * HD, kld = (size_t)Hkv * HD;

  bf16x8_t qf[NKK], dof[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    uint4 a = make_uint4(0, 0, 0, 0), b = make_uint4(0, 0, 0, 0);
    if (qi < L) {
      const size_t o = (size_t)(r0 + qi) * qld + (size_t)h * HD + kk * 16 + g * 8;
      a = *(const uint4 *)(q + o);
      b = *(const uint4 *)(d_o + o);
    }
    qf[kk] = as_bf8(a);
    dof[kk] = as_bf8(b);
  }
  const float sc = 1.4426950408889634f / sqrtf((float)HD), rs = 1.0f / sqrtf((float)HD);
  float lse2 = 0.f, dv_ = 0.f;
  if (qi < L) {
    lse2 = lse[(size_t)(r0 + qi) * Hq + h] * 1.4426950408889634f;
    dv_ = dvec[(size_t)(r0 + qi) * Hq + h];
  }
  f32x16_t acc[NOT];
#pragma unroll
  for (int t = 0; t < NOT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

  const int kend = min(L, q0 + 128);
  const bf16_t *kbase = k + (size_t)r0 * kld + (size_t)kvh * HD, *vbase = v + (size_t)r0 * kld + (size_t)kvh * HD;
  for (int kb = 0; kb < kend; kb += TB) {
    __syncthreads();
    stage_rows<HD>(Ks, kbase, kld, kb, L);
    stage_rows<HD>(Vs, vbase, kld, kb, L);
    stage_rows_t<HD>(Kt, kbase, kld, kb, L);
    __syncthreads();
    if (kb > qw0 + 31) continue;
#pragma unroll
    for (int st = 0; st < 2; ++st) {
      f32x16_t sa, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sa[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        const bf16x8_t a = *(const bf16x8_t *)(Ks + (st * 32 + j) * KP + kk * 16 + g * 8);
        sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], sa, 0, 0, 0);
        const bf16x8_t b = *(const bf16x8_t *)(Vs + (st * 32 + j) * KP + kk * 16 + g * 8);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, dof[kk], dp, 0, 0, 0);
      }
      float ds[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = kb + st * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        const float p = (key <= qi && key < L) ? exp2f(sa[r] * sc - lse2) : 0.f;
        ds[r] = p * (dp[r] - dv_) * rs;
      }
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        const bf16x8_t dsf = pack8(ds + 8 * mm);
#pragma unroll
        for (int t = 0; t < NOT; ++t) {
          const bf16x8_t a = *(const bf16x8_t *)(Kt + (t * 32 + j) * TP + st * 32 + mm * 16 + g * 8);
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, dsf, acc[t], 0, 0, 0);
        }
      }
    }
  }
  if (qi < L) {
    float *dst = dq + (size_t)(r0 + qi) * qld + (size_t)h * HD;
#pragma unroll
    for (int t = 0; t < NOT; ++t)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq)
        *(float4 *)(dst + t * 32 + 8 * rq + 4 * g) = make_float4(acc[t][4 * rq], acc[t][4 * rq + 1], acc[t][4 * rq + 2], acc[t][4 * rq + 3]);
  }
}

// ------------------------------------------------------------------ dK, dV
template <int HD>
__global__ __launch_bounds__(256) void attn_bwd_dkdv_kernel(const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
                                                            const bf16_t *__restrict__ v, const bf16_t *__restrict__ d_o,
                                                            const float *__restrict__ lse, const float *__restrict__ dvec,
                                                            const int32_t *__restrict__ seg, int row_base, int Hq,
                                                            int Hkv, float *__restrict__ dk, float *__restrict__ dv) {
  constexpr int KP = HD + 8, TP = TB + 8, NKK = HD / 16, NOT = HD / 32;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t *Qs = (bf16_t *)smem_raw;          // [TB][KP]
  bf16_t *Os = Qs + TB * KP;                // [TB][KP]   dO rows
  bf16_t *Qt = Os + TB * KP;                // [HD][TP]
  bf16_t *Ot = Qt + HD * TP;                // [HD][TP]   dO transposed
  float *lse_s = (float *)(Ot + HD * TP);   // [TB]  lse * log2(e)
  float *d_s = lse_s + TB;                  // [TB]
  const int s = blockIdx.y, kvh = blockIdx.z, grp = Hq / Hkv;
  const int r0 = seg[s] - row_base, L = seg[s + 1] - seg[s];
  const int k0 = blockIdx.x * 128;
  if (k0 >= L) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, j = lane & 31;
  const int kw0 = k0 + wave * 32, ki = kw0 + j;      // this lane's key
  const size_t qld = (size_t)Hq * HD, kld = (size_t)Hkv * HD;

  bf16x8_t kf[NKK], vf[NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    uint4 a = make_uint4(0, 0, 0, 0), b = make_uint4(0, 0, 0, 0);
    if (ki < L) {
      const size_t o = (size_t)(r0 + ki) * kld + (size_t)kvh * HD + kk * 16 + g * 8;
      a = *(const uint4 *)(k + o);
      b = *(const uint4 *)(v + o);
    }
    kf[kk] = as_bf8(a);
    vf[kk] = as_bf8(b);
  }
  const float sc = 1.4426950408889634f / sqrtf((float)HD), rs = 1.0f / sqrtf((float)HD);
  f32x16_t dka[NOT], dva[NOT];
#pragma unroll
  for (int t = 0; t < NOT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dka[t][r] = 0.f; dva[t][r] = 0.f; }

  for (int gi = 0; gi < grp; ++gi) {
    const int h = kvh * grp + gi;
    const bf16_t *qbase = q + (size_t)r0 * qld + (size_t)h * HD, *obase = d_o + (size_t)r0 * qld + (size_t)h * HD;
    for (int qb = k0; qb < L; qb += TB) {            // k0 is a multiple of 128, so of TB
      __syncthreads();
      stage_rows<HD>(Qs, qbase, qld, qb, L);
      stage_rows<HD>(Os, obase, qld, qb, L);
      stage_rows_t<HD>(Qt, qbase, qld, qb, L);
      stage_rows_t<HD>(Ot, obase, qld, qb, L);
      if (tid < TB) {
        const int qq = qb + tid;
        lse_s[tid] = qq < L ? lse[(size_t)(r0 + qq) * Hq + h] * 1.4426950408889634f : 0.f;
        d_s[tid] = qq < L ? dvec[(size_t)(r0 + qq) * Hq + h] : 0.f;
      }
      __syncthreads();
      if (qb + TB - 1 < kw0) continue;               // every query of the tile precedes this wave's keys
#pragma unroll
      for (int st = 0; st < 2; ++st) {
        f32x16_t sa, dp;
#pragma unroll
        for (int r = 0; r < 16; ++r) { sa[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
        for (int kk = 0; kk < NKK; ++kk) {
          const bf16x8_t a = *(const bf16x8_t *)(Qs + (st * 32 + j) * KP + kk * 16 + g * 8);
          sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kf[kk], sa, 0, 0, 0);
          const bf16x8_t b = *(const bf16x8_t *)(Os + (st * 32 + j) * KP + kk * 16 + g * 8);
          dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, vf[kk], dp, 0, 0, 0);
        }
        float pv[16], ds[16];
#pragma unroll
        for (int rq = 0; rq < 4; ++rq) {
          const float4 l4 = *(const float4 *)(lse_s + st * 32 + 8 * rq + 4 * g);
          const float4 d4 = *(const float4 *)(d_s + st * 32 + 8 * rq + 4 * g);
          const float ll[4] = {l4.x, l4.y, l4.z, l4.w}, dd[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
          for (int e = 0; e < 4; ++e) {
            const int r = 4 * rq + e;
            const int qq = qb + st * 32 + 8 * rq + 4 * g + e;
            const float p = (qq >= ki && qq < L && ki < L) ? exp2f(sa[r] * sc - ll[e]) : 0.f;
            pv[r] = p;
            ds[r] = p * (dp[r] - dd[e]) * rs;
          }
        }
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
          const bf16x8_t pf = pack8(pv + 8 * mm), dsf = pack8(ds + 8 * mm);
#pragma unroll
          for (int t = 0; t < NOT; ++t) {
            const bf16x8_t a = *(const bf16x8_t *)(Ot + (t * 32 + j) * TP + st * 32 + mm * 16 + g * 8);
            dva[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf, dva[t], 0, 0, 0);
            const bf16x8_t b = *(const bf16x8_t *)(Qt + (t * 32 + j) * TP + st * 32 + mm * 16 + g * 8);
            dka[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, dsf, dka[t], 0, 0, 0);
          }
        }
      }
    }
  }
  if (ki < L) {
    float *dkd = dk + (size_t)(r0 + ki) * kld + (size_t)kvh * HD, *dvd = dv + (size_t)(r0 + ki) * kld + (size_t)kvh * HD;
#pragma unroll
    for (int t = 0; t < NOT; ++t)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        *(float4 *)(dkd + t * 32 + 8 * rq + 4 * g) = make_float4(dka[t][4 * rq], dka[t][4 * rq + 1], dka[t][4 * rq + 2], dka[t][4 * rq + 3]);
        *(float4 *)(dvd + t * 32 + 8 * rq + 4 * g) = make_float4(dva[t][4 * rq], dva[t][4 * rq + 1], dva[t][4 * rq + 2], dva[t][4 * rq + 3]);
      }
  }
}

template <int HD>
hipError_t launch_t(const bf16_t *q, const bf16_t *k, const bf16_t *v, const bf16_t *o, const bf16_t *d_o,
                    const float *lse, const int32_t *seg, int row_base, int n_seq, int max_len, int rows, int Hq,
                    int Hkv, float *dvec, float *dq, float *dk, float *dv, hipStream_t st) {
  constexpr size_t lds_q = (size_t)(2 * TB * (HD + 8) + HD * (TB + 8)) * sizeof(bf16_t);
  constexpr size_t lds_k = (size_t)(2 * TB * (HD + 8) + 2 * HD * (TB + 8)) * sizeof(bf16_t) + 2 * TB * sizeof(float);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void *)attn_bwd_dq_kernel<HD>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_q);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)attn_bwd_dkdv_kernel<HD>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_k);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL(attn_dvec_kernel, dim3(rows), dim3(256), 0, st, o, d_o, Hq, HD, dvec);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  dim3 grid_q(cdiv(max_len, 128), n_seq, Hq), grid_k(cdiv(max_len, 128), n_seq, Hkv);
  hipLaunchKernelGGL((attn_bwd_dq_kernel<HD>), grid_q, dim3(256), lds_q, st, q, k, v, d_o, lse, dvec, seg, row_base, Hq, Hkv, dq);
  e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_bwd_dkdv_kernel<HD>), grid_k, dim3(256), lds_k, st, q, k, v, d_o, lse, dvec, seg, row_base, Hq, Hkv, dk, dv);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_bwd(const bf16_t *q, const bf16_t *k, const bf16_t *v, const bf16_t *o, const bf16_t *d_o,
                           const float *lse, const int32_t *seg, int row_base, int n_seq, int max_len, int rows,
                           int Hq, int Hkv, int hd, float *dvec, float *dq, float *dk, float *dv, hipStream_t st) {
  if (n_seq <= 0 || rows <= 0) return hipSuccess;
  if (n_seq > 65535 || Hq > 65535) return hipErrorInvalidValue;
  if (hd == 64) return launch_t<64>(q, k, v, o, d_o, lse, seg, row_base, n_seq, max_len, rows, Hq, Hkv, dvec, dq, dk, dv, st);
  if (hd == 128) return launch_t<128>(q, k, v, o, d_o, lse, seg, row_base, n_seq, max_len, rows, Hq, Hkv, dvec, dq, dk, dv, st);
  return hipErrorInvalidValue;
}
