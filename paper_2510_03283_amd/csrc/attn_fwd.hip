// Varlen causal attention forward on bf16 MFMA (gfx950), for prefill rows (plain bf16 operands)
// and fine-tune rows (two-term bf16 operands, three products per contraction, LSE saved).
//
// One block = 32*NW queries of one (sequence, query head): NW waves x 32 queries.  Scores are
// formed transposed, S^T = K Q^T, so that a lane owns ONE query column: its soft-max state
// (running max, running sum) is a per-lane scalar and P^T is already laid out as the B operand
// of O^T = V^T P^T.  K and V tiles of 64 keys go global -> LDS directly in their memory layout,
// two stages deep (the loads of tile i+1 fly while tile i is multiplied; one barrier per tile);
// K fragments are plain 16-byte LDS reads, V^T fragments come from transposing LDS reads of the
// untransposed V tile (see attn_tile.h).
#include "attn_tile.h"
#include "kernels.h"

namespace {

using namespace attn;

constexpr int KB = 64;    // keys per LDS tile

__device__ __forceinline__ bf16x8_t as_bf8(uint4 u) { return __builtin_bit_cast(bf16x8_t, u); }

// Source of K and V for the PAGED variant (prefill rows of requests with a cached prefix): both
// the prefix and the request's own rows, which the rotary kernel has appended by then, are read
// from the paged cache through the request's block table.
struct PagedKV {
  const bf16_t *cache_k, *cache_v;   // [blocks, Hkv, B, HD] bf16
  const int32_t *block_tables;       // [n_seq, max_blocks]
  const int32_t *prefix_lens;        // [n_seq] cached tokens in front of the request's rows
  long long num_blocks;
  int max_blocks, bshift;
};

template <int HD, bool SPLIT, int NW, bool PAGED>
__global__ __launch_bounds__(64 * NW, NW == 4 ? 2 : 1) void attn_fwd_kernel(const bf16_t *__restrict__ q_hi, const bf16_t *__restrict__ k_hi,
                                                           const bf16_t *__restrict__ v_hi, const bf16_t *__restrict__ q_lo,
                                                           const bf16_t *__restrict__ k_lo, const bf16_t *__restrict__ v_lo,
                                                           const int32_t *__restrict__ seg, int row_base, int Hq, int Hkv,
                                                           bf16_t *__restrict__ o_hi, bf16_t *__restrict__ o_lo,
                                                           float *__restrict__ lse, const PagedKV pg,
                                                           const int32_t *__restrict__ excl_lo, const int32_t *__restrict__ excl_hi) {
  static_assert(!(PAGED && SPLIT), "paged K/V are single bf16 operands");
  constexpr int NT = SPLIT ? 2 : 1;
  constexpr int QB = 32 * NW;
  constexpr int NKK = HD / 16;     // MFMA k-steps over the head dimension
  constexpr int NOT = HD / 32;     // 32-row tiles of O^T
  using T = Tile<KB, HD, 64 * NW>;
  constexpr int STAGE = 2 * NT * T::ELEMS;         // K (hi, lo), V (hi, lo)
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t *lds = (bf16_t *)smem_raw;                // [2][STAGE]

  // blocks are dealt to the XCDs round-robin: block x takes head (x % Hkv) * group + x / Hkv, so the query heads
  // of one kv head (and all their row tiles) run on one XCD and its K and V stay in that XCD's L2
  const int kvh = blockIdx.x % Hkv, h = kvh * (Hq / Hkv) + blockIdx.x / Hkv, s = blockIdx.y;
  const int r0 = seg[s] - row_base, L = seg[s + 1] - seg[s];
  const int q0 = (gridDim.z - 1 - blockIdx.z) * QB;      // long tiles first
  if (q0 >= L) return;
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 5, j = lane & 31;
  const int qw0 = q0 + wave * 32;                        // first query of this wave
  const int qi = qw0 + j;                                // this lane's query (may be >= L: computed, not stored)
  const size_t qld = (size_t)Hq * HD, kld = (size_t)Hkv * HD;
  const bf16_t *kbase[2] = {PAGED ? nullptr : k_hi + (size_t)r0 * kld + (size_t)kvh * HD, SPLIT ? k_lo + (size_t)r0 * kld + (size_t)kvh * HD : nullptr};
  const bf16_t *vbase[2] = {PAGED ? nullptr : v_hi + (size_t)r0 * kld + (size_t)kvh * HD, SPLIT ? v_lo + (size_t)r0 * kld + (size_t)kvh * HD : nullptr};

  // key index space: the request's cached prefix (PAGED only) followed by its own rows
  const int pfx = PAGED ? pg.prefix_lens[s] : 0;
  const int nkeys = pfx + L;
  const int kend = min(nkeys, pfx + q0 + QB);
  const int ntiles = (kend + KB - 1) / KB;
  // optional excluded rectangle: queries >= xhi do not see keys xlo .. xhi-1 (a preference pair stored
  // as prompt | chosen | rejected: the rejected response skips the chosen one)
  const int xlo = excl_lo ? excl_lo[s] : L, xhi = excl_lo ? excl_hi[s] : L;
  auto issue_tile = [&](int it) {
    bf16_t *S = lds + (it & 1) * STAGE;
    if constexpr (PAGED) {
      const int32_t *bt = pg.block_tables + (size_t)s * pg.max_blocks;
      T::issue_paged(pg.cache_k, bt, pg.bshift, Hkv, kvh, pg.num_blocks, it * KB, nkeys, S);
      T::issue_paged(pg.cache_v, bt, pg.bshift, Hkv, kvh, pg.num_blocks, it * KB, nkeys, S + T::ELEMS);
    } else {
#pragma unroll
      for (int t = 0; t < NT; ++t) {
        T::issue(kbase[t], kld, it * KB, L, S + t * T::ELEMS);
        T::issue(vbase[t], kld, it * KB, L, S + (NT + t) * T::ELEMS);
      }
    }
  };
  issue_tile(0);

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

  // lane's K row inside a 32-key sub-tile: MFMA row j reads tile row swap23(j), so that register
  // r = 8*mm + e of S^T holds key 16*mm + 8*g + e
  const typename T::FragK fk = T::frag_k_init(swap23(j));
  typename T::FragT fv[NOT];
#pragma unroll
  for (int t = 0; t < NOT; ++t) fv[t] = T::frag_t_init(32 * t, lane);

  f32x16_t oacc[NOT];
#pragma unroll
  for (int t = 0; t < NOT; ++t)
#pragma unroll
    for (int r = 0; r < 16; ++r) oacc[t][r] = 0.f;
  float m_run = -INFINITY, l_run = 0.f;                  // running max of the raw scores; partial running sum
  const float sc = 1.4426950408889634f / sqrtf((float)HD);

  for (int it = 0; it < ntiles; ++it) {
    wait_vmcnt<0>();
    __syncthreads();                                     // tile it has landed; stage (it+1)&1 is free
    if (it + 1 < ntiles) issue_tile(it + 1);
    const int kb = it * KB;
    if (kb > pfx + qw0 + 31) continue;                   // every key of the tile is in this wave's future
    if (qw0 >= xhi && kb >= xlo && kb + KB <= xhi) continue;   // ... or inside the rectangle this wave must not see
    const bf16_t *Kh = lds + (it & 1) * STAGE, *Kl = Kh + T::ELEMS, *Vh = Kh + NT * T::ELEMS, *Vl = Vh + T::ELEMS;

    // ---- S^T = K Q^T for the two 32-key sub-tiles; lane owns query j, register r owns a key
    f32x16_t sacc[2];
#pragma unroll
    for (int st = 0; st < 2; ++st) {
#pragma unroll
      for (int r = 0; r < 16; ++r) sacc[st][r] = 0.f;
#pragma unroll
      for (int kk = 0; kk < NKK; ++kk) {
        const bf16x8_t a = T::frag_k(Kh + st * 32 * HD, fk, kk, g);
        sacc[st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[0][kk], sacc[st], 0, 0, 0);
        if constexpr (SPLIT) {
          sacc[st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, qf[1][kk], sacc[st], 0, 0, 0);
          const bf16x8_t al = T::frag_k(Kl + st * 32 * HD, fk, kk, g);
          sacc[st] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(al, qf[0][kk], sacc[st], 0, 0, 0);
        }
      }
    }
    // ---- mask (only tiles that touch the diagonal or the end of the sequence), online soft-max
    if (kb + KB - 1 > pfx + qw0 || kb + KB > nkeys || (qw0 + 31 >= xhi && kb < xhi && kb + KB > xlo)) {
#pragma unroll
      for (int st = 0; st < 2; ++st)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int key = kb + st * 32 + 16 * (r >> 3) + 8 * g + (r & 7);
          if (!(key <= pfx + qi && key < nkeys) || (qi >= xhi && key >= xlo && key < xhi)) sacc[st][r] = -INFINITY;
        }
    }
    float mx = sacc[0][0];
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, sacc[st][r]);
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m_run, mx);                // finite from the first tile on (key 0 <= every query)
    const float alpha = __builtin_amdgcn_exp2f((m_run - m_new) * sc);
    m_run = m_new;
    const float mb = m_new * sc;
    float ps = 0.f;
    bf16x8_t pf[NT][2][2];
#pragma unroll
    for (int st = 0; st < 2; ++st)
#pragma unroll
      for (int mm = 0; mm < 2; ++mm) {
        uint32_t wh[4], wl[4];
#pragma unroll
        for (int e = 0; e < 8; e += 2) {
          const float p0 = __builtin_amdgcn_exp2f(fmaf(sacc[st][8 * mm + e], sc, -mb));
          const float p1 = __builtin_amdgcn_exp2f(fmaf(sacc[st][8 * mm + e + 1], sc, -mb));
          ps += p0 + p1;
          if constexpr (SPLIT) split_pk_bf16(p0, p1, wh[e >> 1], wl[e >> 1]);
          else wh[e >> 1] = cvt_pk_bf16(p0, p1);
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
          const bf16x8_t a = T::frag_t(Vh, fv[t], 2 * st + mm);
          oacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[0][st][mm], oacc[t], 0, 0, 0);
          if constexpr (SPLIT) {
            oacc[t] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, pf[1][st][mm], oacc[t], 0, 0, 0);
            const bf16x8_t al = T::frag_t(Vl, fv[t], 2 * st + mm);
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
        uint32_t h0, l0, h1, l1;
        split_pk_bf16(oacc[t][4 * rq] * inv, oacc[t][4 * rq + 1] * inv, h0, l0);
        split_pk_bf16(oacc[t][4 * rq + 2] * inv, oacc[t][4 * rq + 3] * inv, h1, l1);
        const size_t o = ob + t * 32 + 8 * rq + 4 * g;
        *(uint2 *)(o_hi + o) = make_uint2(h0, h1);
        if (o_lo) *(uint2 *)(o_lo + o) = make_uint2(l0, l1);
      }
    if (lse && g == 0) lse[(size_t)(r0 + qi) * Hq + h] = (m_run * sc + log2f(l_tot)) * 0.6931471805599453f;
  }
}

template <int HD, bool SPLIT, int NW, bool PAGED = false>
hipError_t launch_t(const bf16_t *q_hi, const bf16_t *k_hi, const bf16_t *v_hi, const bf16_t *q_lo, const bf16_t *k_lo,
                    const bf16_t *v_lo, const int32_t *seg, int row_base, int n_seq, int max_len, int Hq, int Hkv,
                    bf16_t *o_hi, bf16_t *o_lo, float *lse, hipStream_t st, const PagedKV pg = PagedKV{},
                    const int32_t *excl_lo = nullptr, const int32_t *excl_hi = nullptr) {
  constexpr int NT = SPLIT ? 2 : 1;
  constexpr size_t lds = (size_t)2 * 2 * NT * KB * HD * sizeof(bf16_t);
  static DeviceOnce attr_done;
  if (!attr_done.test()) {
    hipError_t e = hipFuncSetAttribute((const void *)attn_fwd_kernel<HD, SPLIT, NW, PAGED>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done.set();
  }
  dim3 grid(Hq, n_seq, cdiv(max_len, 32 * NW));
  hipLaunchKernelGGL((attn_fwd_kernel<HD, SPLIT, NW, PAGED>), grid, dim3(64 * NW), lds, st, q_hi, k_hi, v_hi, q_lo, k_lo, v_lo, seg, row_base, Hq, Hkv, o_hi, o_lo, lse, pg, excl_lo, excl_hi);
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_fwd(const bf16_t *q_hi, const bf16_t *k_hi, const bf16_t *v_hi, const bf16_t *q_lo,
                           const bf16_t *k_lo, const bf16_t *v_lo, const int32_t *seg, int row_base, int n_seq,
                           int max_len, int Hq, int Hkv, int hd, bf16_t *o_hi, bf16_t *o_lo, float *lse,
                           hipStream_t st, const int32_t *excl_lo, const int32_t *excl_hi) {
  if (n_seq <= 0 || max_len <= 0) return hipSuccess;
  if (n_seq > 65535 || max_len > 65535 * 64 || ((excl_lo == nullptr) != (excl_hi == nullptr))) return hipErrorInvalidValue;
  const bool split = q_lo != nullptr;
  if (split && (!k_lo || !v_lo)) return hipErrorInvalidValue;
  // two-term operands at head dim 128 need 128 KB of LDS per block: 8 waves share it
  if (hd == 64) return split ? launch_t<64, true, 4>(q_hi, k_hi, v_hi, q_lo, k_lo, v_lo, seg, row_base, n_seq, max_len, Hq, Hkv, o_hi, o_lo, lse, st, PagedKV{}, excl_lo, excl_hi)
                             : launch_t<64, false, 4>(q_hi, k_hi, v_hi, q_lo, k_lo, v_lo, seg, row_base, n_seq, max_len, Hq, Hkv, o_hi, o_lo, lse, st, PagedKV{}, excl_lo, excl_hi);
  if (hd == 128) return split ? launch_t<128, true, 8>(q_hi, k_hi, v_hi, q_lo, k_lo, v_lo, seg, row_base, n_seq, max_len, Hq, Hkv, o_hi, o_lo, lse, st, PagedKV{}, excl_lo, excl_hi)
                              : launch_t<128, false, 4>(q_hi, k_hi, v_hi, q_lo, k_lo, v_lo, seg, row_base, n_seq, max_len, Hq, Hkv, o_hi, o_lo, lse, st, PagedKV{}, excl_lo, excl_hi);
  return hipErrorInvalidValue;
}

hipError_t launch_attn_fwd_paged(const bf16_t *q, const void *cache_k, const void *cache_v, long long num_blocks, int block_size,
                                 const int32_t *block_tables, int max_blocks, const int32_t *prefix_lens, const int32_t *seg,
                                 int row_base, int n_seq, int max_len, int Hq, int Hkv, int hd, bf16_t *o, hipStream_t st) {
  if (n_seq <= 0 || max_len <= 0) return hipSuccess;
  if (n_seq > 65535 || max_len > 65535 * 64 || block_size <= 0 || (block_size & (block_size - 1)) || max_blocks <= 0) return hipErrorInvalidValue;
  int bshift = 0;
  while ((1 << bshift) < block_size) ++bshift;
  const PagedKV pg{(const bf16_t *)cache_k, (const bf16_t *)cache_v, block_tables, prefix_lens, num_blocks, max_blocks, bshift};
  if (hd == 64) return launch_t<64, false, 4, true>(q, nullptr, nullptr, nullptr, nullptr, nullptr, seg, row_base, n_seq, max_len, Hq, Hkv, o, nullptr, nullptr, st, pg);
  if (hd == 128) return launch_t<128, false, 4, true>(q, nullptr, nullptr, nullptr, nullptr, nullptr, seg, row_base, n_seq, max_len, Hq, Hkv, o, nullptr, nullptr, st, pg);
  return hipErrorInvalidValue;
}
