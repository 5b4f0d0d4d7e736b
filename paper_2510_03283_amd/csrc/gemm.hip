// bf16 MFMA GEMM for gfx950: 32x32x16 MFMA tiles, direct global->LDS operand loads, LDS double
// buffer of 64-wide k tiles.
//
// Tiles sit in LDS in the layout they have in memory: a k-contiguous operand as [row][k], a
// row-contiguous operand as [k][row].  MFMA fragments (8 consecutive k of one row per lane) come
// from one 16-byte LDS read in the first case and from two transposing 8-byte LDS reads
// (ds_read_b64_tr_b16) in the second, so the NN and TN forms need no transposed copies in HBM
// and no in-register shuffles.
#include "gemm.h"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <type_traits>
#include <utility>
#include <vector>

namespace {

constexpr int BK = 64;          // k extent of an LDS tile
constexpr int NSTAGES = 2;

typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
typedef __attribute__((ext_vector_type(2))) uint32_t u32x2_t;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4_t;   // per-lane byte offsets of up to four tile loads

constexpr int GROUP_M = 8;         // m tiles per swizzle group (L2 reuse of the B tiles)
constexpr int GROUP_M_MULTI = 4;   // the same for row groups with two-term operands (twice the A bytes per m tile)

// Operand tiles go global -> LDS directly (global_load_lds_dwordx4): no staging registers and no
// LDS store instructions.  A wave-wide load writes 64 consecutive 16-byte chunks, so LDS tiles
// are unpadded; bank conflicts are avoided by an XOR swizzle that is applied through the choice
// of the global address each lane fetches.
__device__ __align__(16) uint4 g_zero16 = {0u, 0u, 0u, 0u};   // source of out-of-range chunks

typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void gbl_void_t;

template <int N>
__device__ __forceinline__ void wait_vmcnt() {   // vmcnt <= N, no wait on the other counters
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

template <int ROWS, int LAYOUT, int BKT, int NTHR>
struct DirectStage {
  static constexpr int ELEMS = ROWS * BKT;
  static constexpr int NCH = ROWS * BKT / 8;             // 16-byte chunks
  static constexpr int NI = NCH / NTHR;                  // wave-wide loads per wave
  static_assert(NCH % NTHR == 0 && NI <= 4, "tile must split evenly over the waves, at most four loads per lane");
  static constexpr int CPR = LAYOUT == 0 ? BKT / 8 : ROWS / 8;   // chunks per LDS row
  static constexpr int RPB = LAYOUT == 0 ? 16 / CPR : 1;         // LDS rows per 256 bytes (LAYOUT 0)

  // LAYOUT 0: LDS [row][BKT], chunk position pos holds logical k-chunk pos ^ ((row / RPB) % CPR)
  // LAYOUT 1: LDS [k][ROWS],  logical row-chunk c sits at position c ^ ((k & 3) << 2) when CPR is a
  //           power of two, else at (c + 4 * (k & 3)) % CPR (same bank spread, any CPR % 4 == 0)
  static constexpr bool POW2 = (CPR & (CPR - 1)) == 0;
  static_assert(LAYOUT == 0 || CPR % 4 == 0, "row-contiguous tiles need a multiple of 32 rows");
  static __device__ __forceinline__ void issue(const bf16_t *base, long long ld, int row0, int rows, int k0, int K, bf16_t *S) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int q = wave + (NTHR / 64) * i;
      const int chunk = q * 64 + lane;
      const int lr = chunk / CPR, pos = chunk % CPR;
      const bf16_t *src;
      bool ok;
      if constexpr (LAYOUT == 0) {
        const int kc = pos ^ ((lr / RPB) % CPR);
        const int gr = row0 + lr;
        ok = gr < rows;
        src = base + (long long)gr * ld + k0 + kc * 8;
      } else {
        const int c = POW2 ? pos ^ ((lr & 3) << 2) : (pos + CPR - 4 * (lr & 3)) % CPR;
        const int k = k0 + lr, gr = row0 + 8 * c;
        ok = k < K && gr < rows;
        src = base + (long long)k * ld + gr;
      }
      if (!ok) src = (const bf16_t *)&g_zero16;
      __builtin_amdgcn_global_load_lds((gbl_void_t *)src, (lds_void_t *)(S + q * 512), 16, 0, 0);
    }
  }
  // SwiGLU mode (LAYOUT 0): LDS rows [64 w, 64 w + 32) hold gate rows f0 + 32 w .. and rows
  // [64 w + 32, 64 w + 64) the up rows of the same hidden units, so that the two 32-column MFMA
  // tiles of wave column w are G and U of one unit range.
  static __device__ __forceinline__ void issue_gu(const bf16_t *bg, const bf16_t *bu, long long ld, int f0, int F, int k0, bf16_t *S) {
    static_assert(LAYOUT == 0, "gate/up interleaving is defined for k-contiguous weights");
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int q = wave + (NTHR / 64) * i;
      const int chunk = q * 64 + lane;
      const int lr = chunk / CPR, pos = chunk % CPR;
      const int kc = pos ^ ((lr / RPB) % CPR);
      const int f = f0 + (lr >> 6) * 32 + (lr & 31);
      const bf16_t *src = ((lr >> 5) & 1 ? bu : bg) + (long long)f * ld + k0 + kc * 8;
      if (f >= F) src = (const bf16_t *)&g_zero16;
      __builtin_amdgcn_global_load_lds((gbl_void_t *)src, (lds_void_t *)(S + q * 512), 16, 0, 0);
    }
  }
  // Fast path of the main loop: every lane keeps one 32-bit byte offset per load, relative to a tile
  // origin that is uniform over the block, so a k step costs scalar pointer arithmetic only and the
  // loads take the (scalar base + lane offset) form.  Rows past the matrix edge are clamped onto the
  // last valid row (8-row chunk): they only feed accumulator rows / columns that are never stored.
  // Tiles that cross the end of the k range go through issue() instead (zero fill).
  static __device__ __forceinline__ u32x4_t lane_offsets(long long ld, int row0, int rows, int wave) {
    const int lane = threadIdx.x & 63;
    u32x4_t off = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int chunk = (wave + (NTHR / 64) * i) * 64 + lane;
      const int lr = chunk / CPR, pos = chunk % CPR;
      if constexpr (LAYOUT == 0) {
        const int kc = pos ^ ((lr / RPB) % CPR);
        off[i] = (uint32_t)(((long long)min(lr, rows - 1 - row0) * ld + kc * 8) * 2);
      } else {
        const int c = POW2 ? pos ^ ((lr & 3) << 2) : (pos + CPR - 4 * (lr & 3)) % CPR;
        off[i] = (uint32_t)(((long long)lr * ld + min(8 * c, rows - 8 - row0)) * 2);
      }
    }
    return off;
  }
  static __device__ __forceinline__ u32x4_t lane_offsets_gu(long long ld, int f0, int F, int wave) {
    const int lane = threadIdx.x & 63;
    u32x4_t off = {0u, 0u, 0u, 0u};
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int chunk = (wave + (NTHR / 64) * i) * 64 + lane;
      const int lr = chunk / CPR, pos = chunk % CPR;
      const int kc = pos ^ ((lr / RPB) % CPR);
      const int fr = (lr >> 6) * 32 + (lr & 31);
      off[i] = (uint32_t)(((long long)min(fr, F - 1 - f0) * ld + kc * 8) * 2);
    }
    return off;
  }
  static __device__ __forceinline__ void issue_fast(const char *origin, const u32x4_t off, int wave, bf16_t *S) {
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int q = wave + (NTHR / 64) * i;
      __builtin_amdgcn_global_load_lds((gbl_void_t *)(origin + off[i]), (lds_void_t *)(S + q * 512), 16, 0, 0);
    }
  }
  // SwiGLU mode: a wave-wide load covers 8 LDS rows, so it reads gate rows or up rows, never both
  static __device__ __forceinline__ void issue_fast_gu(const char *origin_g, const char *origin_u, const u32x4_t off, int wave, bf16_t *S) {
    static_assert(LAYOUT == 0 && CPR == 8, "gate/up interleaving is defined for k-contiguous 64-wide tiles");
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int q = wave + (NTHR / 64) * i;
      const char *origin = (q >> 2) & 1 ? origin_u : origin_g;
      __builtin_amdgcn_global_load_lds((gbl_void_t *)(origin + off[i]), (lds_void_t *)(S + q * 512), 16, 0, 0);
    }
  }
  // MFMA fragments (8 consecutive k of one row per lane).  The LDS reads are issued as asm and the
  // kernel counts them itself (s_waitcnt lgkmcnt(n) before the MFMAs that need them): while a direct
  // global->LDS load is in flight the compiler's own wait insertion turns every wait for an LDS
  // read into a wait for ALL outstanding LDS reads, which serialises fragment reads and MFMAs.
  // A read's result must not be touched before that wait; cook() turns it into the MFMA operand.
  static constexpr int RPF = LAYOUT == 0 ? 1 : 2;          // LDS read instructions per fragment
  struct Raw { u32x4_t q; u32x2_t lo, hi; };                // q: k-contiguous tile; lo, hi: transposing reads
  // per-lane byte offsets inside a tile: LAYOUT 0: v[kk] for the lane's first fragment at k step kk
  // (the swizzle depends on kk; fragment i sits i * 32 rows further); LAYOUT 1: v[i] for fragment i
  // at k step 0 (k step kk sits 16 kk rows further)
  struct FragAddr { uint32_t v[4]; };
  template <int NF>
  static __device__ __forceinline__ FragAddr frag_addr(int r0, int lane) {
    static_assert(NF <= 4 && BKT / 16 <= 4, "at most four fragments per wave and four k steps per tile");
    FragAddr f;
#pragma unroll
    for (int x = 0; x < 4; ++x) {
      if constexpr (LAYOUT == 0) {
        const int row = r0 + (lane & 31);
        const int c = (2 * x + (lane >> 5)) ^ ((row / RPB) % CPR);
        f.v[x] = (uint32_t)((row * BKT + c * 8) * 2);
      } else {
        const int grp = lane >> 4, j = lane & 15;
        const int cl = ((r0 + 32 * x) >> 3) + 2 * (grp & 1) + ((j & 3) >> 1);
        const int chunk = POW2 ? cl ^ ((j >> 2) << 2) : (cl + 4 * (j >> 2)) % CPR;
        f.v[x] = x < NF ? (uint32_t)(((8 * (grp >> 1) + (j >> 2)) * ROWS + chunk * 8 + 4 * (j & 1)) * 2) : 0u;
      }
    }
    return f;
  }
  // tile: LDS byte address of the tile; kk, i: compile-time constants at every call site
  static __device__ __forceinline__ Raw read(uint32_t tile, const FragAddr &f, int kk, int i) {
    Raw r;
    if constexpr (LAYOUT == 0) {
      asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(r.q) : "v"(tile + f.v[kk]), "i"(i * 32 * BKT * 2));
    } else {
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.lo) : "v"(tile + f.v[i]), "i"(kk * 16 * ROWS * 2));
      asm volatile("ds_read_b64_tr_b16 %0, %1 offset:%2" : "=v"(r.hi) : "v"(tile + f.v[i]), "i"(kk * 16 * ROWS * 2 + 4 * ROWS * 2));
    }
    return r;
  }
  static __device__ __forceinline__ bf16x8_t cook(const Raw &r) {
    if constexpr (LAYOUT == 0) {
      return __builtin_bit_cast(bf16x8_t, r.q);
    } else {
      const u32x4_t v = {r.lo[0], r.lo[1], r.hi[0], r.hi[1]};
      return __builtin_bit_cast(bf16x8_t, v);
    }
  }
};

template <int N>
__device__ __forceinline__ void wait_lgkmcnt() {   // lgkmcnt <= N, no wait on the other counters
  static_assert(N >= 0 && N <= 15, "4-bit counter");
  __builtin_amdgcn_s_waitcnt(15 | (7 << 4) | (N << 8) | (3 << 14));
}

template <int BM, int BN, int WGM, int WGN, int LA, int LB, int BKT, int NST>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_dl_kernel(const GemmParams p) {
  constexpr int NTHR = 64 * WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;
  constexpr int TM = WTM / 32, TN = WTN / 32;
  constexpr int NKK = BKT / 16;
  constexpr int P = NST - 1;                      // tiles in flight ahead of the one being multiplied
  using SA = DirectStage<BM, LA, BKT, NTHR>;
  using SB = DirectStage<BN, LB, BKT, NTHR>;
  constexpr int STAGE = SA::ELEMS + SB::ELEMS;
  constexpr int LPT = SA::NI + SB::NI;            // loads per thread per tile
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t *lds = (bf16_t *)smem_raw;

  // Block -> tile.  Row groups are laid out one after the other in block-id order (the launcher
  // sorts the multi-pass groups first, so the long tiles start first).  Inside a group, the blocks
  // that land on XCD x (block id % 8) take a contiguous chunk of the group's tile list, ordered in
  // bands of GROUP_M (GROUP_M_MULTI) m-tiles, so the tiles resident on one XCD share A and B panels in its L2 and
  // every XCD gets the same mix of long and short tiles.
  const int n_ns_eff = p.swiglu ? 1 : p.n_ns;      // SwiGLU mode: one logical column range of F hidden units
  const int total_nt = p.nt_start[n_ns_eff];
  int g = 0, first_blk = 0;
  while (g + 1 < p.n_mg && (int)blockIdx.x >= first_blk + (p.mt_start[g + 1] - p.mt_start[g]) * total_nt) {
    first_blk += (p.mt_start[g + 1] - p.mt_start[g]) * total_nt;
    ++g;
  }
  const int mtc = p.mt_start[g + 1] - p.mt_start[g], T = mtc * total_nt;
  int v = 0;
  {
    const int x = blockIdx.x & 7;
    for (int y = 0; y < x; ++y) {
      const int fy = (y - first_blk) & 7;            // first block of the group on XCD y (group-local id)
      v += fy < T ? (T - 1 - fy) / 8 + 1 : 0;
    }
    v += ((int)blockIdx.x - first_blk - ((x - first_blk) & 7)) >> 3;
  }
  const int band = p.mg[g].npass >= 2 ? GROUP_M_MULTI : GROUP_M;
  const int grp_sz = band * total_nt;
  const int first_m = (v / grp_sz) * band;
  const int gm = min(mtc - first_m, band);
  const int mt_l = first_m + (v % grp_sz) % gm, nt_g = (v % grp_sz) / gm;
  int s = 0;
  while (s + 1 < n_ns_eff && nt_g >= p.nt_start[s + 1]) ++s;
  const GemmMGroup &G = p.mg[g];
  const GemmNSeg &S = p.ns[s];
  const int m0 = mt_l * BM, n0 = p.swiglu ? nt_g * (BN / 2) : (nt_g - p.nt_start[s]) * BN;
  const int M = G.M, N = S.N, K = p.K;
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave / WGN, wn = wave % WGN;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  // split-K: grid.y slices the k tiles; slice z writes its partial sums at C + z * c_split_stride
  const int nk_all = (K + BKT - 1) / BKT;
  const int nk_per = (nk_all + (int)gridDim.y - 1) / (int)gridDim.y;
  const int kt0 = (int)blockIdx.y * nk_per;
  const int nk = max(0, min(nk_per, nk_all - kt0));
  const int n_it = nk * G.npass;
  // operand bases of this block's row group / column segment (scalar registers), and every lane's
  // byte offsets inside a tile
  const char *const a_hi = (const char *)G.a[0], *const a_lo = (const char *)G.a[1];
  const char *const b_hi = (const char *)(p.swiglu ? p.ns[0].b[0] : S.b[0]), *const b_lo = (const char *)(p.swiglu ? p.ns[0].b[1] : S.b[1]);
  const char *const u_hi = (const char *)p.ns[1].b[0], *const u_lo = (const char *)p.ns[1].b[1];      // SwiGLU mode: up weights
  const char *const ks_b0 = (const char *)p.kseg_b[0], *const ks_b1 = (const char *)p.kseg_b[1], *const ks_b2 = (const char *)p.kseg_b[2];
  const int ks_s1 = p.kseg_start[1], ks_s2 = p.kseg_start[2];
  const int n_kseg = p.n_kseg, swiglu = p.swiglu;
  const long long lda = p.lda, ldb = p.ldb;
  const u32x4_t offA = SA::lane_offsets(lda, m0, M, wave);
  u32x4_t offB;
  if constexpr (LB == 0) offB = swiglu ? SB::lane_offsets_gu(ldb, n0, N, wave) : SB::lane_offsets(ldb, n0, N, wave);
  else offB = SB::lane_offsets(ldb, n0, N, wave);
  const typename SA::FragAddr fa = SA::template frag_addr<TM>(wm * WTM, lane);
  const typename SB::FragAddr fb = SB::template frag_addr<TN>(wn * WTN, lane);
  const uint32_t lds_addr = (uint32_t)(uintptr_t)(lds_void_t *)lds;      // LDS byte address of stage 0
  constexpr int RPS = TM * SA::RPF + TN * SB::RPF;                       // LDS read instructions per k step
  static_assert(RPS <= 15, "the reads of one k step must fit the 4-bit LDS counter");

  // One loop requests and multiplies: iteration `it` first waits for tile `it`, then requests tile
  // it + P into the stage that tile it - 1 has just left, then multiplies tile `it`.  The first P
  // iterations (it < 0) only request.  (The request code appears once, in line: as a lambda called
  // from two places its captured bases end up in private memory.)
  int st_cur = 0, st_req = 0;
  for (int it = -P; it < n_it; ++it) {
    if (it >= 0) {
      // tile `it` has landed once at most the loads of the P-1 younger tiles are outstanding
      if (it + P - 1 < n_it) wait_vmcnt<(P - 1) * LPT>();
      else wait_vmcnt<0>();
      __syncthreads();   // tile it visible to every wave; every wave is done with the stage of tile it-1
    }
    if (it + P < n_it) {
      const int t = it + P;
      const int pass = t >= 2 * nk ? 2 : (t >= nk ? 1 : 0);
      const int kt = kt0 + t - pass * nk, k0 = kt * BKT;
      bf16_t *st = lds + st_req * STAGE;
      st_req = st_req == NST - 1 ? 0 : st_req + 1;
      if ((LA == 1 || LB == 1) && k0 + BKT > K) {
        // the tile crosses the end of the k range: per-lane bounds checks and zero fill
        SA::issue((const bf16_t *)(pass == 1 ? a_lo : a_hi), lda, m0, M, k0, K, st);
        if (n_kseg > 1) {
          const int ks = (k0 >= ks_s1 ? 1 : 0) + (n_kseg > 2 && k0 >= ks_s2 ? 1 : 0);
          const int s0 = ks == 0 ? 0 : (ks == 1 ? ks_s1 : ks_s2), s1 = ks + 1 == n_kseg ? K : (ks == 0 ? ks_s1 : ks_s2);
          SB::issue((const bf16_t *)(ks == 0 ? ks_b0 : (ks == 1 ? ks_b1 : ks_b2)), ldb, n0, N, k0 - s0, s1 - s0, st + SA::ELEMS);
        } else {
          SB::issue((const bf16_t *)(pass == 2 ? b_lo : b_hi), ldb, n0, N, k0, K, st + SA::ELEMS);
        }
      } else {
        const char *ao = (pass == 1 ? a_lo : a_hi) + (LA == 0 ? (long long)m0 * lda + k0 : (long long)k0 * lda + m0) * 2;
        SA::issue_fast(ao, offA, wave, st);
        if (n_kseg > 1) {
          const int ks = (k0 >= ks_s1 ? 1 : 0) + (n_kseg > 2 && k0 >= ks_s2 ? 1 : 0);
          const int kl = k0 - (ks == 0 ? 0 : (ks == 1 ? ks_s1 : ks_s2));
          const char *bo = (ks == 0 ? ks_b0 : (ks == 1 ? ks_b1 : ks_b2)) + (LB == 0 ? (long long)n0 * ldb + kl : (long long)kl * ldb + n0) * 2;
          SB::issue_fast(bo, offB, wave, st + SA::ELEMS);
        } else if (swiglu) {
          if constexpr (LB == 0) {
            const long long o = ((long long)n0 * ldb + k0) * 2;
            SB::issue_fast_gu((pass == 2 ? b_lo : b_hi) + o, (pass == 2 ? u_lo : u_hi) + o, offB, wave, st + SA::ELEMS);
          }
        } else {
          const char *bo = (pass == 2 ? b_lo : b_hi) + (LB == 0 ? (long long)n0 * ldb + k0 : (long long)k0 * ldb + n0) * 2;
          SB::issue_fast(bo, offB, wave, st + SA::ELEMS);
        }
      }
    }
    if (it < 0) continue;
    const uint32_t Ac = lds_addr + st_cur * (STAGE * 2), Bc = Ac + SA::ELEMS * 2;
    typename SA::Raw ra[2][TM];
    typename SB::Raw rb[2][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i) ra[0][i] = SA::read(Ac, fa, 0, i);
#pragma unroll
    for (int j = 0; j < TN; ++j) rb[0][j] = SB::read(Bc, fb, 0, j);
#pragma unroll
    for (int kk = 0; kk < NKK; ++kk) {
      if (kk + 1 < NKK) {
#pragma unroll
        for (int i = 0; i < TM; ++i) ra[(kk + 1) & 1][i] = SA::read(Ac, fa, kk + 1, i);
#pragma unroll
        for (int j = 0; j < TN; ++j) rb[(kk + 1) & 1][j] = SB::read(Bc, fb, kk + 1, j);
        wait_lgkmcnt<RPS>();          // the fragments of step kk are in; those of step kk + 1 may be in flight
      } else {
        wait_lgkmcnt<0>();
      }
      __builtin_amdgcn_sched_barrier(0);
      bf16x8_t af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = SA::cook(ra[kk & 1][i]);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[j] = SB::cook(rb[kk & 1][j]);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    st_cur = st_cur == NST - 1 ? 0 : st_cur + 1;
  }

  // epilogue: accumulator register r of a 32x32 tile holds row 8*(r/4) + 4*(lane/32) + r%4, column lane%32.
  // bf16 outputs are stored as packed pairs: neighbouring lanes (columns f, f+1) swap one value of
  // a register pair (rows row, row+1), the even lane then stores columns (f, f+1) of row and the
  // odd lane columns (f-1, f) of row+1 - one 4-byte store per lane instead of two 2-byte ones.
  const int rk = p.resid_kind, obf = p.out_bf16;
  const long long ldc = p.ldc, ldr = p.ldr;
  const bool odd = lane & 1;
  auto swap_pair = [&](float mine_r, float mine_r1) -> float {     // returns the partner's value for the row this lane stores
    const float send = odd ? mine_r : mine_r1;
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(send), 0xB1, 0xF, 0xF, true));
  };
  if (p.swiglu) {
    if constexpr (TN == 2 && LB == 0) {
      const int f = n0 + wn * 32 + (lane & 31);
      const int F = N;
      bf16_t *hi = (bf16_t *)G.c, *lo = (bf16_t *)G.c_lo, *gu = (bf16_t *)G.c_gu;
#pragma unroll
      for (int i = 0; i < TM; ++i) {
        const int rbase = m0 + wm * WTM + i * 32 + 4 * (lane >> 5);
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const int row0 = rbase + 8 * (r >> 2) + (r & 3);
          float g2[2] = {acc[i][0][r], acc[i][0][r + 1]}, u2[2] = {acc[i][1][r], acc[i][1][r + 1]}, h2[2];
#pragma unroll
          for (int e = 0; e < 2; ++e) h2[e] = g2[e] / (1.0f + expf(-g2[e])) * u2[e];
          const float hp = swap_pair(h2[0], h2[1]), gp = swap_pair(g2[0], g2[1]), up = swap_pair(u2[0], u2[1]);
          const int row = row0 + (odd ? 1 : 0), fc = f - (odd ? 1 : 0);          // this lane stores (row, fc .. fc+1)
          if (row < M && fc < F) {
            const float ha = odd ? hp : h2[0], hb = odd ? h2[1] : hp;
            uint32_t ph, pl;
            split_pk_bf16(ha, hb, ph, pl);
            *(uint32_t *)(hi + (long long)row * ldc + fc) = ph;
            if (lo) *(uint32_t *)(lo + (long long)row * ldc + fc) = pl;
            if (gu) {
              *(uint32_t *)(gu + (long long)row * 2 * F + fc) = cvt_pk_bf16(odd ? gp : g2[0], odd ? g2[1] : gp);
              *(uint32_t *)(gu + (long long)row * 2 * F + F + fc) = cvt_pk_bf16(odd ? up : u2[0], odd ? u2[1] : up);
            }
          }
        }
      }
    }
    return;
  }
  if (obf && !(N & 1) && !(S.c_col & 1)) {
    // packed bf16 path (every lane takes part in the swap, also those beyond the matrix edge)
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
      for (int j = 0; j < TN; ++j) {
        const int col = n0 + wn * WTN + j * 32 + (lane & 31);
        const int rbase = m0 + wm * WTM + i * 32 + 4 * (lane >> 5);
        const long long cc = S.c_col + col;
#pragma unroll
        for (int r = 0; r < 16; r += 2) {
          const int row0 = rbase + 8 * (r >> 2) + (r & 3);
          float va = acc[i][j][r], vb = acc[i][j][r + 1];
          if (rk && col < N) {
            if (row0 < M) va += rk == 1 ? ((const float *)G.resid)[row0 * ldr + cc] : bf2f(((const bf16_t *)G.resid)[row0 * ldr + cc]);
            if (row0 + 1 < M) vb += rk == 1 ? ((const float *)G.resid)[(row0 + 1) * ldr + cc] : bf2f(((const bf16_t *)G.resid)[(row0 + 1) * ldr + cc]);
          }
          const float vp = swap_pair(va, vb);
          const int row = row0 + (odd ? 1 : 0);
          if (row < M && col - (odd ? 1 : 0) < N)
            *(uint32_t *)((bf16_t *)G.c + row * ldc + cc - (odd ? 1 : 0)) = cvt_pk_bf16(odd ? vp : va, odd ? vb : vp);
        }
      }
    }
    return;
  }
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn * WTN + j * 32 + (lane & 31);
      const int rbase = m0 + wm * WTM + i * 32 + 4 * (lane >> 5);
      if (col >= N) continue;
      const long long cc = S.c_col + col + (long long)blockIdx.y * p.c_split_stride;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = rbase + 8 * (r >> 2) + (r & 3);
        if (row < M) {
          float v = acc[i][j][r];
          if (rk == 1) v += ((const float *)G.resid)[row * ldr + cc];
          else if (rk == 2) v += bf2f(((const bf16_t *)G.resid)[row * ldr + cc]);
          if (obf) ((bf16_t *)G.c)[row * ldc + cc] = f2bf(v);
          else ((float *)G.c)[row * ldc + cc] = v;
        }
      }
    }
  }
}

template <int BM, int BN>
int count_tiles(GemmParams &p) {
  int mt = 0, nt = 0;
  for (int g = 0; g < p.n_mg; ++g) { p.mt_start[g] = mt; mt += cdiv(p.mg[g].M, BM); }
  p.mt_start[p.n_mg] = mt;
  if (p.swiglu) {
    p.nt_start[0] = 0;
    nt = cdiv(p.ns[0].N, BN / 2);
    p.nt_start[1] = nt;
    return mt * nt;
  }
  for (int s = 0; s < p.n_ns; ++s) { p.nt_start[s] = nt; nt += cdiv(p.ns[s].N, BN); }
  p.nt_start[p.n_ns] = nt;
  return mt * nt;
}

#include "gemm_w4.h"

template <int BM, int BN, int WGM, int WGN, int LA, int LB, int BKT, int NST>
hipError_t launch_dl(GemmParams &p, hipStream_t stream) {
  const int tiles = count_tiles<BM, BN>(p);
  if (tiles == 0) return hipSuccess;
  constexpr int NTHR = 64 * WGM * WGN;
  constexpr size_t lds = (size_t)NST * (BM + BN) * BKT * sizeof(bf16_t);
  static_assert(lds <= 160 * 1024, "LDS budget of a gfx950 CU");
  static DeviceOnce attr_done;
  if (!attr_done.test()) {
    hipError_t e = hipFuncSetAttribute((const void *)gemm_bf16_dl_kernel<BM, BN, WGM, WGN, LA, LB, BKT, NST>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done.set();
  }
  p.tile_m = BM; p.tile_n = BN;
  hipLaunchKernelGGL((gemm_bf16_dl_kernel<BM, BN, WGM, WGN, LA, LB, BKT, NST>), dim3((unsigned)tiles, (unsigned)(p.k_splits > 1 ? p.k_splits : 1)), dim3(NTHR), lds, stream, p);
  return hipGetLastError();
}

template <int LA, int LB>
hipError_t launch_w4(GemmParams &p, hipStream_t stream) {
  const int tiles = count_tiles<256, 256>(p);
  if (tiles == 0) return hipSuccess;
  constexpr size_t lds = (size_t)2 * (256 + 256) * BK * sizeof(bf16_t);
  static DeviceOnce attr_done;
  if (!attr_done.test()) {
    hipError_t e = hipFuncSetAttribute((const void *)gemm_bf16_w4_kernel<LA, LB>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done.set();
  }
  p.tile_m = 256; p.tile_n = 256;
  hipLaunchKernelGGL((gemm_bf16_w4_kernel<LA, LB>), dim3((unsigned)tiles, (unsigned)(p.k_splits > 1 ? p.k_splits : 1)), dim3(256), lds, stream, p);
  return hipGetLastError();
}

bool aligned16(const void *q) { return ((uintptr_t)q & 15) == 0; }

// Tile choice.  256x256 tiles (four waves with 128x128 wave tiles, one block per CU) do 0.5 LDS fragment
// reads per MFMA and half the L2 traffic of 128x128 tiles (4 waves, two blocks per CU), but quantise worse on
// small problems; 192x256 (8 waves) sits between.  Each candidate is priced as
//   length of its schedule over the (CU x resident block) slots  x  tile area  /  relative efficiency,
// a tile of a row group with p passes taking p time units on its slot, and the cheapest is launched.  The
// efficiencies (0.69 for 192x256, 0.62 for 128x128, relative to the four-wave kernel) are fitted to whole steps
// of the benchmark configurations: step time is flat for factors between 0.68 and 0.8 of the kernels' long-run
// ratios (0.92, 0.83) and 1 - 6 % worse on either side.
template <int BM, int BN>
double tile_cost(const GemmParams &p, int slots, double slot_share, double eff) {
  const int ks = p.k_splits > 1 ? p.k_splits : 1;
  int nt = 0;
  for (int s = 0; s < p.n_ns; ++s) nt += cdiv(p.ns[s].N, BN);
  // The dispatcher hands the next block to whichever slot is free, in block-id order (row groups one
  // after the other, multi-pass groups first).  Time in passes of one tile: free_at[t] slots fall free at t.
  double w = 0;
  for (int g = 0; g < p.n_mg; ++g) w += (double)cdiv(p.mg[g].M, BM) * nt * p.mg[g].npass * ks;
  std::vector<int> free_at((size_t)(w / slots) + 8, 0);
  free_at[0] = slots;
  size_t t = 0, end = 0;
  for (int g = 0; g < p.n_mg; ++g) {
    long long n = (long long)cdiv(p.mg[g].M, BM) * nt * ks;
    const size_t c = (size_t)p.mg[g].npass;
    while (n > 0) {
      if (free_at[t] == 0) { ++t; continue; }
      const int k = (int)std::min<long long>(n, free_at[t]);
      free_at[t] -= k;
      free_at[t + c] += k;
      n -= k;
      end = std::max(end, t + c);
    }
  }
  return (double)end * BM * BN * slot_share / eff;
}

// 1: 256x256, 2: 192x256, 0: 128x128
int choose_tile(const GemmParams &p) {
  const double c256 = tile_cost<256, 256>(p, 256, 1.0, 1.0);
  const double c192 = tile_cost<192, 256>(p, 256, 1.0, 0.69);
  const double c128 = tile_cost<128, 128>(p, 512, 2.0, 0.62);
  return c256 <= c192 && c256 <= c128 ? 1 : (c192 <= c128 ? 2 : 0);
}

bool has_rope(const GemmParams &p) {
  for (int g = 0; g < p.n_mg; ++g)
    if (p.mg[g].rope) return true;
  return false;
}

template <int LA, int LB>
bool uses_w4(const GemmParams &p) {
  return (p.force_w4 || choose_tile(p) == 1) && w4_fits<LA, LB>(p);
}

template <int LA, int LB>
hipError_t launch_layout(GemmParams &p, hipStream_t stream, const char **why) {
  if (p.force_w4 || p.swiglu_bwd || has_rope(p)) {      // forms that only the four-wave kernel has
    if (!uses_w4<LA, LB>(p)) { *why = "gemm: the problem does not run on the four-wave kernel"; return hipErrorInvalidValue; }
    return launch_w4<LA, LB>(p, stream);
  }
  const int tile = choose_tile(p);
  if (tile == 1) {
    // the four-wave kernel, at every reduction length (measured against the eight-wave kernel of the same tile:
    // 5 % faster at K = 1024 .. 2048, 7 - 12 % at K >= 4096); the eight-wave kernel takes what does not fit it
    if (w4_fits<LA, LB>(p)) return launch_w4<LA, LB>(p, stream);
    return launch_dl<256, 256, 2, 4, LA, LB, BK, NSTAGES>(p, stream);
  }
  if (tile == 2) return launch_dl<192, 256, 2, 4, LA, LB, BK, NSTAGES>(p, stream);
  return launch_dl<128, 128, 2, 2, LA, LB, BK, NSTAGES>(p, stream);
}

}  // namespace

hipError_t gemm_launch(int LA, int LB, GemmParams &p, hipStream_t stream, const char **why) {
  *why = nullptr;
  if (p.n_mg < 1 || p.n_mg > 3 || p.n_ns < 1 || p.n_ns > 3) { *why = "gemm: group count"; return hipErrorInvalidValue; }
  if (p.K <= 0) { *why = "gemm: K <= 0"; return hipErrorInvalidValue; }
  if (p.k_splits > 1 && (p.resid_kind || p.out_bf16 || p.c_split_stride <= 0)) { *why = "gemm: split-K needs fp32 output without residual"; return hipErrorInvalidValue; }
  if ((LA == 0 || LB == 0) && p.K % BK) { *why = "gemm: K of a k-contiguous operand must be a multiple of 64"; return hipErrorInvalidValue; }
  if (p.lda % 8 || p.ldb % 8) { *why = "gemm: leading dimension not a multiple of 8"; return hipErrorInvalidValue; }
  if (p.lda <= 0 || p.ldb <= 0 || p.lda >= (1 << 22) || p.ldb >= (1 << 22)) { *why = "gemm: leading dimension out of range"; return hipErrorInvalidValue; }
  for (int g = 0; g < p.n_mg; ++g) {
    const GemmMGroup &G = p.mg[g];
    if (G.M < 0 || G.npass < 1 || G.npass > 3) { *why = "gemm: bad row group"; return hipErrorInvalidValue; }
    if (G.M == 0) continue;
    if (!G.a[0] || !aligned16(G.a[0]) || !G.c) { *why = "gemm: A/C pointer"; return hipErrorInvalidValue; }
    if (G.npass >= 2 && (!G.a[1] || !aligned16(G.a[1]))) { *why = "gemm: A lo pointer"; return hipErrorInvalidValue; }
    if (LA == 1 && G.M % 8) { *why = "gemm: M of an m-contiguous operand must be a multiple of 8"; return hipErrorInvalidValue; }
    if (p.resid_kind && !G.resid) { *why = "gemm: residual pointer"; return hipErrorInvalidValue; }
    for (int s = 0; s < p.n_ns; ++s)
      if (G.npass == 3 && !p.ns[s].b[1]) { *why = "gemm: B lo pointer"; return hipErrorInvalidValue; }
  }
  for (int s = 0; s < p.n_ns; ++s) {
    const GemmNSeg &S = p.ns[s];
    if (S.N <= 0 || !S.b[0] || !aligned16(S.b[0]) || (S.b[1] && !aligned16(S.b[1]))) { *why = "gemm: bad column segment"; return hipErrorInvalidValue; }
    if (LB == 1 && S.N % 8) { *why = "gemm: N of an n-contiguous operand must be a multiple of 8"; return hipErrorInvalidValue; }
  }
  if (p.out_bf16 && p.ldc % 2) { *why = "gemm: bf16 output needs an even leading dimension"; return hipErrorInvalidValue; }
  if (p.swiglu) {
    if (LA != 0 || LB != 0 || p.n_ns != 2 || p.ns[0].N != p.ns[1].N || p.ns[0].N % 2 || p.k_splits > 1 || p.resid_kind || p.n_kseg > 1 || p.ldc % 2) {
      *why = "gemm: SwiGLU mode needs the NT form, two equal column segments and a plain bf16 output";
      return hipErrorInvalidValue;
    }
  }
  if (has_rope(p)) {
    bool ok = LA == 0 && LB == 0 && !p.swiglu && !p.swiglu_bwd && !p.out_bf16 && !p.resid_kind && p.k_splits <= 1 && p.n_kseg <= 1 && p.rope_cs;
    for (int s = 0; s < p.n_ns; ++s) ok = ok && p.ns[s].N % 128 == 0 && p.ns[s].rope_hi;
    if (!ok) { *why = "gemm: rotary mode needs the NT form, plain fp32 output for the other rows, segments of whole 128-wide heads and an angle table"; return hipErrorInvalidValue; }
  }
  if (p.swiglu_bwd) {
    if (LA != 0 || LB != 1 || p.n_ns != 1 || p.ns[0].c_col != 0 || p.ns[0].N % 2 || !p.out_bf16 || p.resid_kind || p.k_splits > 1 || p.swiglu ||
        p.ldc != 2ll * p.ns[0].N) {
      *why = "gemm: SwiGLU backward mode needs the NN form, one column segment, bf16 output [M, 2N] and no residual";
      return hipErrorInvalidValue;
    }
    for (int g = 0; g < p.n_mg; ++g)
      if (!p.mg[g].c_gu) { *why = "gemm: SwiGLU backward mode needs G | U of the forward"; return hipErrorInvalidValue; }
  }
  if (p.n_kseg > 1) {
    if (p.n_kseg > 3 || p.n_ns != 1 || p.kseg_start[0] != 0 || p.kseg_start[p.n_kseg] != p.K) { *why = "gemm: bad k segments"; return hipErrorInvalidValue; }
    for (int g = 0; g < p.n_mg; ++g)
      if (p.mg[g].npass != 1) { *why = "gemm: k segments need single-pass row groups"; return hipErrorInvalidValue; }
    for (int s = 0; s < p.n_kseg; ++s)
      if (!p.kseg_b[s] || !aligned16(p.kseg_b[s]) || p.kseg_start[s] % BK || p.kseg_start[s + 1] <= p.kseg_start[s]) { *why = "gemm: bad k segment"; return hipErrorInvalidValue; }
  }
  // multi-pass row groups first (stable): their tiles take longest and should start first
  for (int i = 1; i < p.n_mg; ++i)
    for (int j = i; j > 0 && p.mg[j].npass > p.mg[j - 1].npass; --j) std::swap(p.mg[j], p.mg[j - 1]);
  if (LA == 0 && LB == 0) return launch_layout<0, 0>(p, stream, why);
  if (LA == 0 && LB == 1) return launch_layout<0, 1>(p, stream, why);
  if (LA == 1 && LB == 1) return launch_layout<1, 1>(p, stream, why);
  *why = "gemm: unsupported layout";
  return hipErrorInvalidValue;
}

bool gemm_uses_four_wave(int LA, int LB, const GemmParams &p) {
  if (LA == 0 && LB == 0) return uses_w4<0, 0>(p);
  if (LA == 0 && LB == 1) return uses_w4<0, 1>(p);
  if (LA == 1 && LB == 1) return uses_w4<1, 1>(p);
  return false;
}

int gemm_suggest_k_splits(int M, int N, int K) {
  const int nk = cdiv(K, BK);
  if (nk < 32) return 1;
  GemmParams p;
  memset(&p, 0, sizeof(p));
  p.n_mg = p.n_ns = 1;
  p.mg[0].M = M; p.mg[0].npass = 1;
  p.ns[0].N = N;
  // seconds: a CU does about 3.5 TFLOP/s on a 256x256 tile; partial sums move at about 3 TB/s
  double best = 0;
  int best_ks = 1;
  for (int ks = 1; ks <= 8; ++ks) {
    if (nk / ks < 16) break;
    p.k_splits = ks;
    const double c = std::min(std::min(tile_cost<256, 256>(p, 256, 1.0, 1.0), tile_cost<192, 256>(p, 256, 1.0, 0.92)),
                              tile_cost<128, 128>(p, 512, 2.0, 0.83));
    double t = c * 2.0 * ((double)K / ks) / 3.5e12;
    if (ks > 1) t += 4e-6 + (double)(ks + 1) * M * N * 4.0 / 3e12;
    if (ks == 1 || t < best * 0.95) { best = t; best_ks = ks; }
  }
  return best_ks;
}
