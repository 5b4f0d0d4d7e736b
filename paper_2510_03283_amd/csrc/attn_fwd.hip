// Varlen causal attention forward on bf16 MFMA (gfx950), for prefill rows (plain bf16 operands)
// and fine-tune rows (two-term bf16 operands, three products per contraction, LSE saved).
//
// One block = 128 queries of one (sequence, query head): 4 waves x 32 queries.  Scores are formed
// transposed, S^T = K Q^T, so that a lane owns ONE query column: its soft-max state (running
// max, running sum) is a per-lane scalar and P^T is already laid out as the B operand of
// O^T = V^T P^T.  K tiles sit in LDS as [key][hd]; V tiles are transposed on the way in to
// [hd][key'] with key' = key with bits 2 and 3 swapped, which makes the 8 keys a lane needs for
// one MFMA contiguous (one 16-byte LDS read).
#include "kernels.h"

namespace {

constexpr int QB = 128;   // queries per block
constexpr int KB = 64;    // keys per LDS tile

__device__ __forceinline__ bf16x8_t as_bf8(uint4 u) { return __builtin_bit_cast(bf16x8_t, u); }

template <int HD, bool SPLIT>
__global__ __launch_bounds__(256) void attn_fwd_kernel(const bf16_t *__restrict__ q_hi, const bf16_t *__restrict__ k_hi,
                                                       const bf16_t *__restrict__ v_hi, const bf16_t *__restrict__ q_lo,
                                                       const bf16_t *__restrict__ k_lo, const bf16_t *__restrict__ v_lo,
                                                       const int32_t *__restrict__ seg, int row_base, int Hq, int Hkv,
                                                       bf16_t *__restrict__ o_hi, bf16_t *__restrict__ o_lo,
                                                       float *__restrict__ lse) {
  constexpr int NT = SPLIT ? 2 : 1;
  constexpr int KP = HD + 8;       // pitch of a K row in LDS
  constexpr int VP = KB + 8;       // pitch of a V^T row in LDS
  constexpr int NKK = HD / 16;     // MFMA k-steps over the head dimension
  constexpr int NOT = HD / 32;     // 32-row tiles of O^T
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t *Ks = (bf16_t *)smem_raw;                 // [NT][KB][KP]
  bf16_t *Vt = Ks + NT * KB * KP;                  // [NT][HD][VP]

  const int s = blockIdx.y, h = blockIdx.z, kvh = h / (Hq / Hkv);
  const int r0 = seg[s] - row_base, L = seg[s + 1] - seg[s];
  const int q0 = (gridDim.x - 1 - blockIdx.x) * QB;      // long tiles first
  if (q0 >= L) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, j = lane & 31;
  const int qw0 = q0 + wave * 32;                        // first query of this wave
  const int qi = qw0 + j;                                // this lane's query (may be >= L: computed, not stored)
  const size_t qld = (size_t)Hq * HD, kld = (size_t)Hkv * HD;

  // Q fragments (B operand of S^T): 8 consecutive head-dim elements per k-step, kept in registers
  bf16x8_t qf[NT][NKK];
#pragma unroll
  for (int kk = 0; kk < NKK; ++kk) {
    uint4 vh = make_uint4(0, 0, 0, 0), vl = make_uint4(0, 0, 0, 0);
    if (qi < L) {
      const size_t o = (size_t)(r0 + qi) * qld + (size_t)h * HD + kk * 16 + g * 8;
      vh = *(const uint4 *)(q_hi + o);
      if constexpr (SPLIT) vl = *(const uint4 *)(q_lo + o);
    }
    qf[0][kk] = as_bf8(vh);
    if constexpr (SPLIT) qf[1][kk] = as_bf8(vl);
  }

  f32x16_t oacc[NOT];
#pragma unroll
  for (int t = 0; t < NOT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[t][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;                  // log2-domain running max; partial running sum
  const float sc = 1.4426950408889634f / sqrtf((float)HD);

  const int kend = min(L, q0 + QB);
  for (int kb = 0; kb < kend; kb += KB) {
    __syncthreads();
    // ---- stage K tile [key][hd] and V tile transposed [hd][key']
#pragma unroll
    for (int t = 0; t < NT; ++t) {
      const bf16_t *kp = t ? k_lo : k_hi;
      const bf16_t *vp = t ? v_lo : v_hi;
      for (int c = tid; c < KB * HD / 8; c += 256) {
        const int key = c / (HD / 8), ch = c % (HD / 8);
        uint4 v = make_uint4(0, 0, 0, 0);
        if (kb + key < L) v = *(const uint4 *)(kp + (size_t)(r0 + kb + key) * kld + (size_t)kvh * HD + ch * 8);
        *(uint4 *)(Ks + (t * KB + key) * KP + ch * 8) = v;
      }
      for (int c = tid; c < (KB / 4) * (HD / 8); c += 256) {
        const int hb = c % (HD / 8), kq = c / (HD / 8);           // 8 head-dim elements x 4 keys
        uint32_t d[4][4];
#pragma unroll
        for (int jj = 0; jj < 4; ++jj) {
          uint4 v = make_uint4(0, 0, 0, 0);
          const int key = kb + 4 * kq + jj;
          if (key < L) v = *(const uint4 *)(vp + (size_t)(r0 + key) * kld + (size_t)kvh * HD + hb * 8);
          d[jj][0] = v.x; d[jj][1] = v.y; d[jj][2] = v.z; d[jj][3] = v.w;
        }
        const int kq2 = (kq & ~3) | ((kq & 1) << 1) | ((kq >> 1) & 1);   // swap key bits 2 and 3
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
          *(uint2 *)(Vt + (t * HD + hb * 8 + m) * VP + 4 * kq2) = make_uint2(w0, w1);
        }
      }
    }
    __syncthreads();
    if (kb > qw0 + 31) continue;                         // every key of the tile is in this wave's future

    // ---- S^T = K Q^T for the two 32-key sub-tiles; lane owns query j, register r owns key
    f32x16_t sacc[2];
#pragma unroll
    for (int st = 0; st < 2; ++st) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[st][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        const bf16x8_t a = *(const bf16x8_t *)(Ks + (st * 32 + j) * KP + kk * 16 + g * 8);
        sacc[st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[0][kk], sacc[st], 0, 0, 0);
        if constexpr (SPLIT) {
          sacc[st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[1][kk], sacc[st], 0, 0, 0);
          const bf16x8_t al = *(const bf16x8_t *)(Ks + (KB + st * 32 + j) * KP + kk * 16 + g * 8);
          sacc[st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, qf[0][kk], sacc[st], 0, 0, 0);
        }
      }
    }
    // ---- mask, online soft-max (log2 domain)
    float mx = -INFINITY;
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int key = kb + st * 32 + 8 * (r >> 2) + 4 * g + (r & 3);
        const float t = (key <= qi && key < L) ? sacc[st][r] * sc : -INFINITY;
        sacc[st][r] = t;
        mx = fmaxf(mx, t);
      }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);                // finite from the first tile on (key 0 <= every query)
    const float alpha = exp2f(m_run - m_new);
    m_run = m_new;
    float ps = 0.f;
    bf16x8_t pf[NT][2][2];
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        uint32_t wh[4], wl[4];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const float p0 = exp2f(sacc[st][8 * mm + e] - m_new), p1 = exp2f(sacc[st][8 * mm + e + 1] - m_new);
          ps += p0 + p1;
          bf16_t h0, l0, h1, l1;
          split_bf(p0, h0, l0);
          split_bf(p1, h1, l1);
          wh[e >> 1] = pack2(h0, h1);
          wl[e >> 1] = pack2(l0, l1);
        }
        pf[0][st][mm] = as_bf8(make_uint4(wh[0], wh[1], wh[2], wh[3]));
        if constexpr (SPLIT) pf[1][st][mm] = as_bf8(make_uint4(wl[0], wl[1], wl[2], wl[3]));
      }
    l_run = l_run * alpha + ps;
    // ---- O^T = alpha O^T + V^T P^T
#pragma unroll
    for (int t = 0; t < NOT; ++t) {
#pragma unroll
      for (int r = 0; r < 16; ++r) oacc[t][r] *= alpha;
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
          const bf16x8_t a = *(const bf16x8_t *)(Vt + (t * 32 + j) * VP + st * 32 + mm * 16 + g * 8);
          oacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[0][st][mm], oacc[t], 0, 0, 0);
          if constexpr (SPLIT) {
            oacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[1][st][mm], oacc[t], 0, 0, 0);
            const bf16x8_t al = *(const bf16x8_t *)(Vt + (HD + t * 32 + j) * VP + st * 32 + mm * 16 + g * 8);
            oacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, pf[0][st][mm], oacc[t], 0, 0, 0);
          }
        }
    }
  }

  // ---- normalise and store: lane owns query qi, rows 32t + 8(r/4) + 4g + r%4 of O^T
  const float l_tot = l_run + __shfl_xor(l_run, 32, 64);
  if (qi < L) {
    const float inv = 1.0f / l_tot;
    const size_t ob = (size_t)(r0 + qi) * qld + (size_t)h * HD;
#pragma unroll
    for (int t = 0; t < NOT; ++t)
#pragma unroll
      for (int rq = 0; rq < 4; ++rq) {
        bf16_t hh[4], ll[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) split_bf(oacc[t][4 * rq + e] * inv, hh[e], ll[e]);
        const size_t o = ob + t * 32 + 8 * rq + 4 * g;
        *(uint2 *)(o_hi + o) = make_uint2(pack2(hh[0], hh[1]), pack2(hh[2], hh[3]));
        if (o_lo) *(uint2 *)(o_lo + o) = make_uint2(pack2(ll[0], ll[1]), pack2(ll[2], ll[3]));
      }
    if (lse && g == 0) lse[(size_t)(r0 + qi) * Hq + h] = (m_run + log2f(l_tot)) * 0.6931471805599453f;
  }
}

template <int HD, bool SPLIT>
hipError_t launch_t(const bf16_t *q_hi, const bf16_t *k_hi, const bf16_t *v_hi, const bf16_t *q_lo, const bf16_t *k_lo,
                    const bf16_t *v_lo, const int32_t *seg, int row_base, int n_seq, int max_len, int Hq, int Hkv,
                    bf16_t *o_hi, bf16_t *o_lo, float *lse, hipStream_t st) {
  constexpr int NT = SPLIT ? 2 : 1;
  constexpr size_t lds = (size_t)NT * (KB * (HD + 8) + HD * (KB + 8)) * sizeof(bf16_t);
  static bool attr_done = false;
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void *)attn_fwd_kernel<HD, SPLIT>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  dim3 grid(cdiv(max_len, QB), n_seq, Hq);
  hipLaunchKernelGGL((attn_fwd_kernel<HD, SPLIT>), grid, dim3(256), lds, st, q_hi, k_hi, v_hi, q_lo, k_lo, v_lo, seg, row_base, Hq, Hkv, o_hi, o_lo, lse);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_fwd(const bf16_t *q_hi, const bf16_t *k_hi, const bf16_t *v_hi, const bf16_t *q_lo,
                           const bf16_t *k_lo, const bf16_t *v_lo, const int32_t *seg, int row_base, int n_seq,
                           int max_len, int Hq, int Hkv, int hd, bf16_t *o_hi, bf16_t *o_lo, float *lse,
                           hipStream_t st) {
  if (n_seq <= 0 || max_len <= 0) return hipSuccess;
  if (n_seq > 65535 || Hq > 65535) return hipErrorInvalidValue;
  const bool split = q_lo != nullptr;
  if (split && (!k_lo || !v_lo)) return hipErrorInvalidValue;
  if (hd == 64) return split ? launch_t<64, true>(q_hi, k_hi, v_hi, q_lo, k_lo, v_lo, seg, row_base, n_seq, max_len, Hq, Hkv, o_hi, o_lo, lse, st)
                             : launch_t<64, false>(q_hi, k_hi, v_hi, q_lo, k_lo, v_lo, seg, row_base, n_seq, max_len, Hq, Hkv, o_hi, o_lo, lse, st);
  if (hd == 128) return split ? launch_t<128, true>(q_hi, k_hi, v_hi, q_lo, k_lo, v_lo, seg, row_base, n_seq, max_len, Hq, Hkv, o_hi, o_lo, lse, st)
                              : launch_t<128, false>(q_hi, k_hi, v_hi, q_lo, k_lo, v_lo, seg, row_base, n_seq, max_len, Hq, Hkv, o_hi, o_lo, lse, st);
  return hipErrorInvalidValue;
}
