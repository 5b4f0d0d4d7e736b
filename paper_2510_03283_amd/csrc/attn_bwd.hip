// Backward of the varlen causal attention of the fine-tune sequences (bf16 MFMA, fp32 outputs).
//
// Two kernels, each free of atomics and of cross-lane transposes:
//  * dq kernel:  a wave owns 32 queries (a lane owns one query column of S^T = K Q^T and of
//    dP^T = V dO^T), walks the keys, and accumulates dQ^T = K^T dS^T.
//  * dkdv kernel: a wave owns 32 keys (a lane owns one key column of S = Q K^T and dP = dO V^T),
//    walks the queries of every query head of its GQA group, and accumulates
//    dV^T = dO^T P and dK^T = Q^T dS.
// P is recomputed from the saved log-sum-exp; D = rowsum(dO * O) is formed by the dq kernel from the
// fragments it loads anyway and handed to the dk/dv kernel through memory.
// The backward of the rotary embedding is part of both epilogues: the two halves (i, i + hd/2) of a
// head row sit in one lane (accumulator tiles t and t + hd/64), so dq and dk are rotated back by the
// row's angles (a per-row (cos, sin) table) and written, like dv, as bf16 straight into the
// [rows, (Hq + 2 Hkv) hd] operand of the projection backward - no fp32 dq / dk / dv in memory.
// Tiles of 64 rows go global -> LDS directly in their memory layout, two stages deep; the same
// tile feeds the products that reduce over the head dimension (16-byte reads) and those that
// reduce over the tile rows (transposing reads), see attn_tile.h.
#include "attn_tile.h"
#include "kernels.h"

namespace {

using namespace attn;

constexpr int TB = 64;    // rows per staged LDS tile

__device__ __forceinline__ bf16x8_t as_bf8(uint4 u) { return __builtin_bit_cast(bf16x8_t, u); }

__device__ __forceinline__ bf16x8_t pack8(const float *v) {
  return as_bf8(make_uint4(cvt_pk_bf16(v[0], v[1]), cvt_pk_bf16(v[2], v[3]), cvt_pk_bf16(v[4], v[5]), cvt_pk_bf16(v[6], v[7])));
}

// Epilogue of a gradient row held as NOT accumulator tiles of 32 head-dim indices (register 4*rq + e of
// tile t = index 32 t + 8 rq + 4 g + e): rotate the pairs (i, i + HD/2) back by the row's angles
// (cs = (cos, sin) of the row, HD/2 entries; null = no rotation) and store as bf16 at dst[0 .. HD).
template <int HD>
__device__ __forceinline__ void store_grad_row(const f32x16_t (&acc)[HD / 32], const float2 *__restrict__ cs, int g, bf16_t *__restrict__ dst) {
  constexpr int NOT = HD / 32, HT = NOT / 2;
#pragma unroll
  for (int t = 0; t < HT; ++t)
#pragma unroll
    for (int rq = 0; rq < 4; ++rq) {
      const int i = t * 32 + 8 * rq + 4 * g;
      float a[4], b[4];
#pragma unroll
      for (int e = 0; e < 4; ++e) { a[e] = acc[t][4 * rq + e]; b[e] = acc[t + HT][4 * rq + e]; }
      if (cs) {
        const float4 c01 = *(const float4 *)(cs + i), c23 = *(const float4 *)(cs + i + 2);
        const float co[4] = {c01.x, c01.z, c23.x, c23.z}, si[4] = {c01.y, c01.w, c23.y, c23.w};
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          const float ra = a[e] * co[e] + b[e] * si[e], rb = b[e] * co[e] - a[e] * si[e];
          a[e] = ra; b[e] = rb;
        }
      }
      *(uint2 *)(dst + i) = make_uint2(cvt_pk_bf16(a[0], a[1]), cvt_pk_bf16(a[2], a[3]));
      *(uint2 *)(dst + i + HD / 2) = make_uint2(cvt_pk_bf16(b[0], b[1]), cvt_pk_bf16(b[2], b[3]));
    }
}

// ------------------------------------------------------------------ dQ
template <int HD>
__global__ __launch_bounds__(256, 2) void attn_bwd_dq_kernel(const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
                                                          const bf16_t *__restrict__ v, const bf16_t *__restrict__ o,
                                                          const bf16_t *__restrict__ d_o,
                                                          const float *__restrict__ lse, float *__restrict__ dvec,
                                                          const int32_t *__restrict__ seg, int row_base, int Hq, int Hkv,
                                                          const float2 *__restrict__ cs, bf16_t *__restrict__ dqkv,
                                                          const int32_t *__restrict__ excl_lo,
                                                          const int32_t *__restrict__ excl_hi) {
  constexpr int NKK = HD / 16, NOT = HD / 32;
  using T = Tile<TB, HD, 256>;
  constexpr int STAGE = 2 * T::ELEMS;       // K tile, V tile
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t *lds = (bf16_t *)smem_raw;         // [2][STAGE]
  // blocks are dealt to the XCDs round-robin: block x takes head (x % Hkv) * group + x / Hkv, so the query heads
  // of one kv head (and all their row tiles) run on one XCD and its K and V stay in that XCD's L2
  const int kvh = blockIdx.x % Hkv, h = kvh * (Hq / Hkv) + blockIdx.x / Hkv, s = blockIdx.y;
  const int r0 = seg[s] - row_base, L = seg[s + 1] - seg[s];
  const int q0 = (gridDim.z - 1 - blockIdx.z) * 128;
  if (q0 >= L) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, j = lane & 31;
  const int qw0 = q0 + wave * 32, qi = qw0 + j;
  const size_t qld = (size_t)Hq * HD, kld = (size_t)Hkv * HD;
  const bf16_t *kbase = k + (size_t)r0 * kld + (size_t)kvh * HD, *vbase = v + (size_t)r0 * kld + (size_t)kvh * HD;
  const int kend = min(L, q0 + 128);
  const int ntiles = (kend + TB - 1) / TB;
  const int xlo = excl_lo ? excl_lo[s] : L, xhi = excl_lo ? excl_hi[s] : L;   // queries >= xhi skip keys xlo .. xhi-1
  auto issue_tile = [&](int it) {
    bf16_t *S = lds + (it & 1) * STAGE;
    T::issue(kbase, kld, it * TB, L, S);
    T::issue(vbase, kld, it * TB, L, S + T::ELEMS);
  };
  issue_tile(0);

  // q and dO fragments of this lane's query; D = rowsum(dO * O) is formed on the way (each lane of the pair
  // (j, j + 32) holds half of the row) and written out for the dk/dv kernel
  bf16x8_t qf[NKK], dof[NKK];
  float dpart = 0.f;
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    uint4 a = make_uint4(0, 0, 0, 0), b = make_uint4(0, 0, 0, 0), c = make_uint4(0, 0, 0, 0);
    if (qi < L) {
      const size_t off = (size_t)(r0 + qi) * qld + (size_t)h * HD + kk * 16 + g * 8;
      a = *(const uint4 *)(q + off);
      b = *(const uint4 *)(d_o + off);
      c = *(const uint4 *)(o + off);
    }
    qf[kk] = as_bf8(a);
    dof[kk] = as_bf8(b);
    const uint32_t bw[4] = {b.x, b.y, b.z, b.w}, cw[4] = {c.x, c.y, c.z, c.w};
#pragma unroll
    for (int e = 0; e < 4; ++e)
      dpart += __uint_as_float(bw[e] << 16) * __uint_as_float(cw[e] << 16) +
               __uint_as_float(bw[e] & 0xffff0000u) * __uint_as_float(cw[e] & 0xffff0000u);
  }
  const float dv_ = dpart + __shfl_xor(dpart, 32);
  const float sc = 1.4426950408889634f / sqrtf((float)HD), rs = 1.0f / sqrtf((float)HD);
  float lse2 = 0.f;
  if (qi < L) {
    lse2 = lse[(size_t)(r0 + qi) * Hq + h] * 1.4426950408889634f;
    if (g == 0) dvec[(size_t)(r0 + qi) * Hq + h] = dv_;
  }
  // MFMA row j reads tile row swap23(j): register r = 8*mm + e then holds key 16*mm + 8*g + e
  const typename T::FragK fk = T::frag_k_init(swap23(j));
  typename T::FragT ft[NOT];
#pragma unroll
  for (int t = 0; t < NOT; ++t) ft[t] = T::frag_t_init(32 * t, lane);
  f32x16_t acc[NOT];
#pragma unroll
  for (int t = 0; t < NOT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[t][r] = 0.f;

  for (int it = 0; it < ntiles; ++it) {
    wait_vmcnt<0>();
    __syncthreads();                                     // tile it has landed; the other stage is free
    if (it + 1 < ntiles) issue_tile(it + 1);
    const int kb = it * TB;
    if (kb > qw0 + 31) continue;
    if (qw0 >= xhi && kb >= xlo && kb + TB <= xhi) continue;
    const bf16_t *Ks = lds + (it & 1) * STAGE, *Vs = Ks + T::ELEMS;
    const bool need_mask = kb + TB - 1 > qw0 || kb + TB > L || (qw0 + 31 >= xhi && kb < xhi && kb + TB > xlo);
#pragma unroll
    for (int st = 0; st < 2; ++st) {
      f32x16_t sa, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sa[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        const bf16x8_t a = T::frag_k(Ks + st * 32 * HD, fk, kk, g);
        sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[kk], sa, 0, 0, 0);
        const bf16x8_t b = T::frag_k(Vs + st * 32 * HD, fk, kk, g);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, dof[kk], dp, 0, 0, 0);
      }
      float ds[16];
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        float p = __builtin_amdgcn_exp2f(fmaf(sa[r], sc, -lse2));
        if (need_mask) {
          const int key = kb + st * 32 + 16 * (r >> 3) + 8 * g + (r & 7);
          if (!(key <= qi && key < L) || (qi >= xhi && key >= xlo && key < xhi)) p = 0.f;
        }
        ds[r] = p * (dp[r] - dv_) * rs;
      }
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        const bf16x8_t dsf = pack8(ds + 8 * mm);
#pragma unroll
        for (int t = 0; t < NOT; ++t) {
          const bf16x8_t a = T::frag_t(Ks, ft[t], 2 * st + mm);
          acc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, dsf, acc[t], 0, 0, 0);
        }
      }
    }
  }
  if (qi < L)
    store_grad_row<HD>(acc, cs + (size_t)(r0 + qi) * (HD / 2), g, dqkv + (size_t)(r0 + qi) * (qld + 2 * kld) + (size_t)h * HD);
}

// ------------------------------------------------------------------ dK, dV
template <int HD>
__global__ __launch_bounds__(256, HD == 64 ? 2 : 1) void attn_bwd_dkdv_kernel(const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
                                                            const bf16_t *__restrict__ v, const bf16_t *__restrict__ d_o,
                                                            const float *__restrict__ lse, const float *__restrict__ dvec,
                                                            const int32_t *__restrict__ seg, int row_base, int Hq,
                                                            int Hkv, const float2 *__restrict__ cs, bf16_t *__restrict__ dqkv,
                                                            const int32_t *__restrict__ excl_lo, const int32_t *__restrict__ excl_hi) {
  constexpr int NKK = HD / 16, NOT = HD / 32;
  using T = Tile<TB, HD, 256>;
  constexpr int STAGE = 2 * T::ELEMS + 4 * TB;    // Q tile, dO tile, lse[TB] and D[TB] as fp32 (2 bf16 slots each)
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t *lds = (bf16_t *)smem_raw;               // [2][STAGE]
  const int kvh = blockIdx.x, s = blockIdx.y, grp = Hq / Hkv;
  const int r0 = seg[s] - row_base, L = seg[s + 1] - seg[s];
  const int k0 = blockIdx.z * 128;
  if (k0 >= L) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, j = lane & 31;
  const int kw0 = k0 + wave * 32, ki = kw0 + j;      // this lane's key
  const size_t qld = (size_t)Hq * HD, kld = (size_t)Hkv * HD;
  const int xlo = excl_lo ? excl_lo[s] : L, xhi = excl_lo ? excl_hi[s] : L;   // queries >= xhi skip keys xlo .. xhi-1
  const int nqt = (L - k0 + TB - 1) / TB;            // query tiles per head (k0 is a multiple of TB)
  const int niter = grp * nqt;
  auto issue_tile = [&](int it) {
    const int gi = it / nqt, qb = k0 + (it % nqt) * TB;
    const int h = kvh * grp + gi;
    bf16_t *S = lds + (it & 1) * STAGE;
    T::issue(q + (size_t)r0 * qld + (size_t)h * HD, qld, qb, L, S);
    T::issue(d_o + (size_t)r0 * qld + (size_t)h * HD, qld, qb, L, S + T::ELEMS);
    if (wave < 2) {                                  // one 4-byte element per lane: lane's value lands at base + 4*lane
      const int qq = qb + lane;
      const float *src = wave ? dvec : lse;
      const float *p = qq < L ? src + (size_t)(r0 + qq) * Hq + h : (const float *)&zero16;
      __builtin_amdgcn_global_load_lds((gbl_void_t *)p, (lds_void_t *)(S + 2 * T::ELEMS + wave * 2 * TB), 4, 0, 0);
    }
  };
  issue_tile(0);

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
  // MFMA row j reads tile row swap23(j): register r = 8*mm + e then holds query 16*mm + 8*g + e
  const typename T::FragK fk = T::frag_k_init(swap23(j));
  typename T::FragT ft[NOT];
#pragma unroll
  for (int t = 0; t < NOT; ++t) ft[t] = T::frag_t_init(32 * t, lane);
  f32x16_t dka[NOT], dva[NOT];
#pragma unroll
  for (int t = 0; t < NOT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) { dka[t][r] = 0.f; dva[t][r] = 0.f; }

  for (int it = 0; it < niter; ++it) {
    wait_vmcnt<0>();
    __syncthreads();                                 // tile it has landed; the other stage is free
    if (it + 1 < niter) issue_tile(it + 1);
    const int qb = k0 + (it % nqt) * TB;
    if (qb + TB - 1 < kw0) continue;                 // every query of the tile precedes this wave's keys
    if (kw0 >= xlo && kw0 + 32 <= xhi && qb >= xhi) continue;   // ... or none of them may see these keys
    const bf16_t *Qs = lds + (it & 1) * STAGE, *Os = Qs + T::ELEMS;
    const float *lse_s = (const float *)(Os + T::ELEMS), *d_s = lse_s + TB;
    const bool need_mask = qb < kw0 + 31 || qb + TB > L || kw0 + 32 > L || (kw0 + 31 >= xlo && kw0 < xhi && qb + TB > xhi);
#pragma unroll
    for (int st = 0; st < 2; ++st) {
      f32x16_t sa, dp;
#pragma unroll
      for (int r = 0; r < 16; ++r) { sa[r] = 0.f; dp[r] = 0.f; }
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        const bf16x8_t a = T::frag_k(Qs + st * 32 * HD, fk, kk, g);
        sa = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, kf[kk], sa, 0, 0, 0);
        const bf16x8_t b = T::frag_k(Os + st * 32 * HD, fk, kk, g);
        dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, vf[kk], dp, 0, 0, 0);
      }
      float pv[16], ds[16];
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        const int qo = st * 32 + 16 * mm + 8 * g;    // first of the 8 queries in registers 8*mm .. 8*mm+7
        const float4 la = *(const float4 *)(lse_s + qo), lb = *(const float4 *)(lse_s + qo + 4);
        const float4 da = *(const float4 *)(d_s + qo), db = *(const float4 *)(d_s + qo + 4);
        const float ll[8] = {la.x, la.y, la.z, la.w, lb.x, lb.y, lb.z, lb.w};
        const float dd[8] = {da.x, da.y, da.z, da.w, db.x, db.y, db.z, db.w};
#pragma unroll
        for (int e = 0; e < 8; ++e) {
          const int r = 8 * mm + e;
          float p = __builtin_amdgcn_exp2f(fmaf(sa[r], sc, -1.4426950408889634f * ll[e]));
          if (need_mask) {
            const int qq = qb + qo + e;
            if (!(qq >= ki && qq < L && ki < L) || (qq >= xhi && ki >= xlo && ki < xhi)) p = 0.f;
          }
          pv[r] = p;
          ds[r] = p * (dp[r] - dd[e]) * rs;
        }
      }
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        const bf16x8_t pf = pack8(pv + 8 * mm), dsf = pack8(ds + 8 * mm);
#pragma unroll
        for (int t = 0; t < NOT; ++t) {
          const bf16x8_t a = T::frag_t(Os, ft[t], 2 * st + mm);
          dva[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf, dva[t], 0, 0, 0);
          const bf16x8_t b = T::frag_t(Qs, ft[t], 2 * st + mm);
          dka[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(b, dsf, dka[t], 0, 0, 0);
        }
      }
    }
  }
  if (ki < L) {
    bf16_t *row = dqkv + (size_t)(r0 + ki) * (qld + 2 * kld) + qld + (size_t)kvh * HD;     // dk of this kv head; dv sits kld further
    store_grad_row<HD>(dka, cs + (size_t)(r0 + ki) * (HD / 2), g, row);
    store_grad_row<HD>(dva, nullptr, g, row + kld);
  }
}

template <int HD>
hipError_t launch_t(const bf16_t *q, const bf16_t *k, const bf16_t *v, const bf16_t *o, const bf16_t *d_o,
                    const float *lse, const int32_t *seg, int row_base, int n_seq, int max_len, int rows, int Hq,
                    int Hkv, float *dvec, const float2 *cs, bf16_t *dqkv, hipStream_t st, const int32_t *excl_lo,
                    const int32_t *excl_hi) {
  constexpr size_t lds_q = (size_t)2 * (2 * TB * HD) * sizeof(bf16_t);
  constexpr size_t lds_k = (size_t)2 * (2 * TB * HD + 4 * TB) * sizeof(bf16_t);
  static DeviceOnce attr_done;
  if (!attr_done.test()) {
    hipError_t e = hipFuncSetAttribute((const void *)attn_bwd_dq_kernel<HD>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_q);
    if (e != hipSuccess) return e;
    e = hipFuncSetAttribute((const void *)attn_bwd_dkdv_kernel<HD>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds_k);
    if (e != hipSuccess) return e;
    attr_done.set();
  }
  dim3 grid_q(Hq, n_seq, cdiv(max_len, 128)), grid_k(Hkv, n_seq, cdiv(max_len, 128));
  hipLaunchKernelGGL((attn_bwd_dq_kernel<HD>), grid_q, dim3(256), lds_q, st, q, k, v, o, d_o, lse, dvec, seg, row_base, Hq, Hkv, cs, dqkv, excl_lo, excl_hi);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL((attn_bwd_dkdv_kernel<HD>), grid_k, dim3(256), lds_k, st, q, k, v, d_o, lse, dvec, seg, row_base, Hq, Hkv, cs, dqkv, excl_lo, excl_hi);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_bwd(const bf16_t *q, const bf16_t *k, const bf16_t *v, const bf16_t *o, const bf16_t *d_o,
                           const float *lse, const int32_t *seg, int row_base, int n_seq, int max_len, int rows,
                           int Hq, int Hkv, int hd, float *dvec, const float2 *cs, bf16_t *dqkv, hipStream_t st,
                           const int32_t *excl_lo, const int32_t *excl_hi) {
  if (n_seq <= 0 || rows <= 0) return hipSuccess;
  if (n_seq > 65535 || max_len > 65535 * 64 || ((excl_lo == nullptr) != (excl_hi == nullptr))) return hipErrorInvalidValue;
  if (hd == 64) return launch_t<64>(q, k, v, o, d_o, lse, seg, row_base, n_seq, max_len, rows, Hq, Hkv, dvec, cs, dqkv, st, excl_lo, excl_hi);
  if (hd == 128) return launch_t<128>(q, k, v, o, d_o, lse, seg, row_base, n_seq, max_len, rows, Hq, Hkv, dvec, cs, dqkv, st, excl_lo, excl_hi);
  return hipErrorInvalidValue;
}
