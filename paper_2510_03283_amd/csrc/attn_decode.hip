// Decode attention: one query row per request against its paged context, HBM-bound.
//
// Split-KV: grid (kv head, split, request); a block streams `chunk` tokens of one (request, kv head)
// once, for all query heads of the GQA group, with 16-byte loads per lane (a token row of hd
// elements is covered by hd/8 consecutive lanes, so a wave load touches whole token rows that
// are contiguous inside a cache block).  Every lane keeps its own online soft-max state over the
// tokens it sees; states are merged across lanes, waves and finally splits.  bf16 caches use packed
// dot products (v_dot2_f32_bf16) for q.k, DPP row operations for the per-token reduction and
// nontemporal loads (the cache is read once per iteration and should not displace the weights).
#include "kernels.h"

#include <cstdlib>

namespace {

constexpr int MIN_CHUNK = 512, MAX_CHUNK = 4096;   // tokens per block: a power of two in this range, chosen per launch
constexpr int UNR = 4;       // token loads in flight per lane for K and for V

__device__ __forceinline__ float safe_scale(float m_old, float m_new) {
  return m_old == -INFINITY ? 0.f : exp2f(m_old - m_new);
}

// Sum over the LPT (8 or 16) consecutive lanes that share a token row, result in every lane, with
// DPP row operations (quad swaps, then mirrors inside 8 and 16 lanes) - no LDS traffic.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float x) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(x), CTRL, 0xF, 0xF, true));
}
template <int LPT>
__device__ __forceinline__ float group_sum(float d) {
  d += dpp_mov<0xB1>(d);                         // quad_perm [1,0,3,2]
  d += dpp_mov<0x4E>(d);                         // quad_perm [2,3,0,1]
  d += dpp_mov<0x141>(d);                        // row_half_mirror: the other quad of the 8 lanes
  if constexpr (LPT == 16) d += dpp_mov<0x140>(d);   // row_mirror: the other half of the 16 lanes
  return d;
}

typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4_t;
__device__ __forceinline__ float dot2_bf16(uint32_t a, uint32_t b, float c) {
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, a), __builtin_bit_cast(bf16x2_t, b), c, false);
}

// FAST: block_size >= tokens per wave-wide load, so the tokens of one load share a cache block
// and the block-table entry is read once per load (wave-uniform) instead of once per lane.
template <int HD, int GRP, bool CBF, bool FAST>
__global__ __launch_bounds__(256) void attn_decode_kernel(const bf16_t *__restrict__ q, const void *__restrict__ ck,
                                                          const void *__restrict__ cv, long long num_blocks, int B,
                                                          int bshift, const int32_t *__restrict__ block_tables,
                                                          int max_blocks, const int32_t *__restrict__ ctx_lens, int Hq,
                                                          int Hkv, int nsplit, int chunk, float *__restrict__ partial) {
  constexpr int LPT = HD / 8;          // lanes per token row
  constexpr int TPL = 64 / LPT;        // tokens per wave-wide load
  constexpr int NW = CBF ? 4 : 8;      // 32-bit words of the 8 elements a lane holds
  __shared__ float sm[4][GRP][HD + 2];
  const int kvh = blockIdx.x, split = blockIdx.y, req = blockIdx.z;
  const int n_tot = ctx_lens[req] + 1;                    // cached context plus the new token
  const int c0 = split * chunk;
  if (c0 >= n_tot) return;
  const int c1 = min(n_tot, c0 + chunk);
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int e0 = (lane % LPT) * 8, tl = lane / LPT;
  const float sc = 1.4426950408889634f / sqrtf((float)HD);

  // q: packed bf16 pairs for the bf16 cache (dot2), scaled floats for the fp32 cache
  uint32_t qp[GRP][4];
  float qv[GRP][8];
#pragma unroll
  for (int gi = 0; gi < GRP; ++gi) {
    const uint4 u = *(const uint4 *)(q + (size_t)req * Hq * HD + (size_t)(kvh * GRP + gi) * HD + e0);
    qp[gi][0] = u.x; qp[gi][1] = u.y; qp[gi][2] = u.z; qp[gi][3] = u.w;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      qv[gi][2 * e] = __uint_as_float(qp[gi][e] << 16);
      qv[gi][2 * e + 1] = __uint_as_float(qp[gi][e] & 0xffff0000u);
    }
  }
  float m[GRP], l[GRP], acc[GRP][8];
#pragma unroll
  for (int gi = 0; gi < GRP; ++gi) {
    m[gi] = -INFINITY; l[gi] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[gi][e] = 0.f;
  }

  const int32_t *bt = block_tables + (size_t)req * max_blocks;
  const int wbeg = c0 + wave * (chunk / 4), wend = min(c1, wbeg + chunk / 4);
  for (int tb = wbeg; tb < wend; tb += UNR * TPL) {
    long long off[UNR];
    bool ok[UNR];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      const int t0 = tb + u * TPL, t = t0 + tl;
      ok[u] = t < wend;
      long long blk = 0;
      if constexpr (FAST) {
        // t0 is a multiple of TPL <= B: the TPL tokens sit in one block, t0 < wend holds for the first lanes
        blk = t0 < wend ? __builtin_amdgcn_readfirstlane(bt[t0 >> bshift]) : -1;
      } else if (ok[u]) {
        blk = bt[t >> bshift];
      }
      ok[u] = ok[u] && blk >= 0 && blk < num_blocks;      // a bad table entry is ignored, never dereferenced
      off[u] = ok[u] ? ((blk * Hkv + kvh) * B + (t & (B - 1))) * (long long)HD + e0 : 0;
    }
    uint32_t kr[UNR][NW], vr[UNR][NW];
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      if constexpr (CBF) {
        const u32x4_t a = __builtin_nontemporal_load((const u32x4_t *)((const bf16_t *)ck + off[u]));   // streamed once
        kr[u][0] = a.x; kr[u][1] = a.y; kr[u][2] = a.z; kr[u][3] = a.w;
      } else {
        const uint4 a = *(const uint4 *)((const float *)ck + off[u]), b2 = *(const uint4 *)((const float *)ck + off[u] + 4);
        kr[u][0] = a.x; kr[u][1] = a.y; kr[u][2] = a.z; kr[u][3] = a.w; kr[u][4] = b2.x; kr[u][5] = b2.y; kr[u][6] = b2.z; kr[u][7] = b2.w;
      }
    }
#pragma unroll
    for (int u = 0; u < UNR; ++u) {
      if constexpr (CBF) {
        const u32x4_t a = __builtin_nontemporal_load((const u32x4_t *)((const bf16_t *)cv + off[u]));
        vr[u][0] = a.x; vr[u][1] = a.y; vr[u][2] = a.z; vr[u][3] = a.w;
      } else {
        const uint4 a = *(const uint4 *)((const float *)cv + off[u]), b2 = *(const uint4 *)((const float *)cv + off[u] + 4);
        vr[u][0] = a.x; vr[u][1] = a.y; vr[u][2] = a.z; vr[u][3] = a.w; vr[u][4] = b2.x; vr[u][5] = b2.y; vr[u][6] = b2.z; vr[u][7] = b2.w;
      }
    }
    float vf[UNR][8];
#pragma unroll
    for (int u = 0; u < UNR; ++u)
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if constexpr (CBF) vf[u][e] = __uint_as_float((e & 1) ? (vr[u][e >> 1] & 0xffff0000u) : (vr[u][e >> 1] << 16));
        else vf[u][e] = __uint_as_float(vr[u][e]);
      }
#pragma unroll
    for (int gi = 0; gi < GRP; ++gi) {
      float sv[UNR];
      float mx = m[gi];
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        float d = 0.f;
        if constexpr (CBF) {
#pragma unroll
          for (int e = 0; e < 4; ++e) d = dot2_bf16(kr[u][e], qp[gi][e], d);
        } else {
#pragma unroll
          for (int e = 0; e < 8; ++e) d += __uint_as_float(kr[u][e]) * qv[gi][e];
        }
        d = group_sum<LPT>(d) * sc;
        sv[u] = ok[u] ? d : -INFINITY;
        mx = fmaxf(mx, sv[u]);
      }
      if (mx == -INFINITY) continue;                // nothing valid seen yet by this lane group
      const float alpha = safe_scale(m[gi], mx);
      m[gi] = mx;
      l[gi] *= alpha;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[gi][e] *= alpha;
#pragma unroll
      for (int u = 0; u < UNR; ++u) {
        const float p = exp2f(sv[u] - mx);          // exp2(-inf) = 0 for ignored tokens
        l[gi] += p;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[gi][e] += p * vf[u][e];
      }
    }
  }

  // merge the TPL lane groups of the wave (lanes with equal e0)
#pragma unroll
  for (int gi = 0; gi < GRP; ++gi) {
#pragma unroll
    for (int o = LPT; o < 64; o <<= 1) {
      const float m2 = __shfl_xor(m[gi], o, 64), l2 = __shfl_xor(l[gi], o, 64);
      const float mn = fmaxf(m[gi], m2);
      const float a1 = safe_scale(m[gi], mn), a2 = safe_scale(m2, mn);
      l[gi] = l[gi] * a1 + l2 * a2;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[gi][e] = acc[gi][e] * a1 + __shfl_xor(acc[gi][e], o, 64) * a2;
      m[gi] = mn;
    }
    if (lane < LPT) {
#pragma unroll
      for (int e = 0; e < 8; ++e) sm[wave][gi][e0 + e] = acc[gi][e];
      if (lane == 0) { sm[wave][gi][HD] = m[gi]; sm[wave][gi][HD + 1] = l[gi]; }
    }
  }
  __syncthreads();
  // merge the 4 waves; thread t handles (gi, e) pairs
  for (int idx = tid; idx < GRP * HD; idx += 256) {
    const int gi = idx / HD, e = idx - gi * HD;
    float mn = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) mn = fmaxf(mn, sm[w][gi][HD]);
    float lo = 0.f, ao = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float a = safe_scale(sm[w][gi][HD], mn);
      lo += sm[w][gi][HD + 1] * a;
      ao += sm[w][gi][e] * a;
    }
    float *dst = partial + (((size_t)req * Hq + (kvh * GRP + gi)) * nsplit + split) * (HD + 2);
    dst[e] = ao;
    if (e == 0) { dst[HD] = mn; dst[HD + 1] = lo; }
  }
}

template <int HD>
__global__ __launch_bounds__(HD) void attn_decode_combine_kernel(const float *__restrict__ partial,
                                                                 const int32_t *__restrict__ ctx_lens, int Hq, int nsplit, int chunk,
                                                                 bf16_t *__restrict__ out, float *__restrict__ norms) {
  const int req = blockIdx.x, h = blockIdx.y, e = threadIdx.x;
  const int ns = min(nsplit, (ctx_lens[req] + 1 + chunk - 1) / chunk);
  const float *src = partial + ((size_t)req * Hq + h) * nsplit * (HD + 2);
  float mn = -INFINITY;
  for (int s = 0; s < ns; ++s) mn = fmaxf(mn, src[s * (HD + 2) + HD]);
  float lo = 0.f, ao = 0.f;
  for (int s = 0; s < ns; ++s) {
    const float a = safe_scale(src[s * (HD + 2) + HD], mn);
    lo += src[s * (HD + 2) + HD + 1] * a;
    ao += src[s * (HD + 2) + e] * a;
  }
  const float v = lo > 0.f ? ao / lo : 0.f;
  out[((size_t)req * Hq + h) * HD + e] = f2bf(v);
  if (norms) {                                   // L2 norm of the head's output vector (fp32 values)
    __shared__ float red[2];
    float s = wave_sum(v * v);
    if constexpr (HD > 64) {
      if ((e & 63) == 0) red[e >> 6] = s;
      __syncthreads();
      s = red[0] + red[1];
    }
    if (e == 0) norms[(size_t)req * Hq + h] = sqrtf(s);
  }
}

template <int HD, int GRP, bool CBF>
void launch_main(const bf16_t *q, const void *ck, const void *cv, long long num_blocks, int B, int bshift,
                 const int32_t *bt, int max_blocks, const int32_t *ctx, int n_decode, int Hq, int Hkv, int nsplit, int chunk,
                 float *partial, hipStream_t st) {
  if (B >= 64 / (HD / 8))
    hipLaunchKernelGGL((attn_decode_kernel<HD, GRP, CBF, true>), dim3(Hkv, nsplit, n_decode), dim3(256), 0, st, q, ck, cv, num_blocks, B, bshift, bt, max_blocks, ctx, Hq, Hkv, nsplit, chunk, partial);
  else
    hipLaunchKernelGGL((attn_decode_kernel<HD, GRP, CBF, false>), dim3(Hkv, nsplit, n_decode), dim3(256), 0, st, q, ck, cv, num_blocks, B, bshift, bt, max_blocks, ctx, Hq, Hkv, nsplit, chunk, partial);
}

template <int HD, bool CBF>
bool launch_grp(int grp, const bf16_t *q, const void *ck, const void *cv, long long num_blocks, int B, int bshift,
                const int32_t *bt, int max_blocks, const int32_t *ctx, int n_decode, int Hq, int Hkv, int nsplit, int chunk,
                float *partial, hipStream_t st) {
  switch (grp) {
    case 1: launch_main<HD, 1, CBF>(q, ck, cv, num_blocks, B, bshift, bt, max_blocks, ctx, n_decode, Hq, Hkv, nsplit, chunk, partial, st); return true;
    case 2: launch_main<HD, 2, CBF>(q, ck, cv, num_blocks, B, bshift, bt, max_blocks, ctx, n_decode, Hq, Hkv, nsplit, chunk, partial, st); return true;
    case 4: launch_main<HD, 4, CBF>(q, ck, cv, num_blocks, B, bshift, bt, max_blocks, ctx, n_decode, Hq, Hkv, nsplit, chunk, partial, st); return true;
    case 8: launch_main<HD, 8, CBF>(q, ck, cv, num_blocks, B, bshift, bt, max_blocks, ctx, n_decode, Hq, Hkv, nsplit, chunk, partial, st); return true;
    default: return false;
  }
}

}  // namespace

// Tokens per block.  Long chunks mean fewer blocks that find nothing to do, fewer partial states to write
// and merge and a longer stream per block (6.2 -> 6.6 TB/s from 512 to 2048 tokens on a 256-request,
// 32-head batch) - as long as the grid still fills the chip several times over.  Shorter chunks than 512
// tokens do not help small batches (32 requests x 8 kv heads of 4 query heads each: 41 us at 512, 49 us
// at 128): with four query heads per kv head the per-token arithmetic, not the stream, sets the time.
static int decode_chunk_tokens(int n_decode, int Hkv, int max_context, int chunk_tokens) {
  if (chunk_tokens) return chunk_tokens >= MIN_CHUNK && chunk_tokens <= MAX_CHUNK && !(chunk_tokens & (chunk_tokens - 1)) ? chunk_tokens : -1;
  int chunk = MIN_CHUNK;
  while (chunk < MAX_CHUNK && (long long)Hkv * n_decode * cdiv(max_context + 1, 2 * chunk) >= 8192) chunk *= 2;
  return chunk;
}

size_t decode_partial_floats(int n_decode, int Hq, int Hkv, int hd, int max_context, int chunk_tokens) {
  int chunk = decode_chunk_tokens(n_decode, Hkv, max_context, chunk_tokens);
  if (chunk < 0) chunk = MIN_CHUNK;                                    // an invalid override is rejected at launch; size for the worst case
  const size_t nsplit = (size_t)cdiv(max_context + 1, chunk);
  return (size_t)n_decode * Hq * nsplit * (hd + 2);
}

hipError_t launch_attn_decode(const bf16_t *q, const void *cache_k, const void *cache_v, bool cache_bf16,
                              long long num_blocks, int block_size, const int32_t *block_tables, int max_blocks_per_req,
                              const int32_t *ctx_lens, int n_decode, int max_context, int Hq, int Hkv, int hd,
                              float *partial, bf16_t *out, float *norms, hipStream_t st, int chunk_tokens) {
  if (n_decode <= 0) return hipSuccess;
  if (n_decode > 65535 || Hkv > 65535 || Hq > 65535) return hipErrorInvalidValue;
  int bshift = 0;
  while ((1 << bshift) < block_size) ++bshift;
  if ((1 << bshift) != block_size) return hipErrorInvalidValue;
  const int chunk = decode_chunk_tokens(n_decode, Hkv, max_context, chunk_tokens);
  if (chunk < 0) return hipErrorInvalidValue;
  const int nsplit = cdiv(max_context + 1, chunk);
  if (nsplit > 65535) return hipErrorInvalidValue;
  const int grp = Hq / Hkv;
  bool ok = false;
  if (hd == 64) ok = cache_bf16 ? launch_grp<64, true>(grp, q, cache_k, cache_v, num_blocks, block_size, bshift, block_tables, max_blocks_per_req, ctx_lens, n_decode, Hq, Hkv, nsplit, chunk, partial, st)
                                : launch_grp<64, false>(grp, q, cache_k, cache_v, num_blocks, block_size, bshift, block_tables, max_blocks_per_req, ctx_lens, n_decode, Hq, Hkv, nsplit, chunk, partial, st);
  else if (hd == 128) ok = cache_bf16 ? launch_grp<128, true>(grp, q, cache_k, cache_v, num_blocks, block_size, bshift, block_tables, max_blocks_per_req, ctx_lens, n_decode, Hq, Hkv, nsplit, chunk, partial, st)
                                      : launch_grp<128, false>(grp, q, cache_k, cache_v, num_blocks, block_size, bshift, block_tables, max_blocks_per_req, ctx_lens, n_decode, Hq, Hkv, nsplit, chunk, partial, st);
  if (!ok) return hipErrorInvalidValue;
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  if (hd == 64) hipLaunchKernelGGL((attn_decode_combine_kernel<64>), dim3(n_decode, Hq), dim3(64), 0, st, partial, ctx_lens, Hq, nsplit, chunk, out, norms);
  else hipLaunchKernelGGL((attn_decode_combine_kernel<128>), dim3(n_decode, Hq), dim3(128), 0, st, partial, ctx_lens, Hq, nsplit, chunk, out, norms);
  return hipGetLastError();
}
