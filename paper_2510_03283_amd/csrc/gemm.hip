// bf16 MFMA GEMM for gfx950: 32x32x16 MFMA tiles, LDS double buffer, 64-wide k tiles.
//
// Operand tiles are staged global -> registers -> LDS with 16-byte accesses in the layout they
// have in memory: a k-contiguous operand as [row][k], a row-contiguous operand as [k][row].
// MFMA fragments (8 consecutive k of one row per lane) come from one 16-byte LDS read in the
// first case and from two transposing 8-byte LDS reads (ds_read_b64_tr_b16) in the second, so
// the NN and TN forms need no transposed copies in HBM and no in-register shuffles.
#include "gemm.h"

namespace {

constexpr int BK = 64;          // k extent of an LDS tile

typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;

// Global -> register -> LDS staging of one operand tile of ROWS rows (m or n) by BK.
// LAYOUT 0: memory [row][k];  LDS [ROWS][BK + 8]   (pitch 144 B: 16-byte fragment reads conflict-free)
// LAYOUT 1: memory [k][row];  LDS [BK][ROWS + 32]  (pitch = 64 B mod 256 B: 4 k-rows of a transposing read hit disjoint banks)
template <int ROWS, int LAYOUT, int NTHR>
struct TileStage {
  static constexpr int PITCH = LAYOUT == 0 ? BK + 8 : ROWS + 32;
  static constexpr int ELEMS = LAYOUT == 0 ? ROWS * PITCH : BK * PITCH;   // per stage
  static constexpr int NCH = ROWS * BK / 8;            // 16-byte chunks of the tile
  static constexpr int NV = (NCH + NTHR - 1) / NTHR;   // chunks per thread
  static constexpr int CPR = LAYOUT == 0 ? BK / 8 : ROWS / 8;   // chunks per memory row
  uint4 r[NV];

  // rows: valid extent of the row index; K: valid extent of k (only checked for LAYOUT 1, where k is a token count)
  __device__ __forceinline__ void load(const bf16_t *base, long long ld, int row0, int rows, int k0, int K) {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = threadIdx.x + NTHR * i;
      uint4 v = make_uint4(0, 0, 0, 0);
      if (NCH % NTHR == 0 || c < NCH) {
        if constexpr (LAYOUT == 0) {
          const int gr = row0 + c / CPR;
          if (gr < rows) v = *(const uint4 *)(base + (long long)gr * ld + k0 + (c % CPR) * 8);
        } else {
          const int k = k0 + c / CPR, gr = row0 + (c % CPR) * 8;
          if (k < K && gr < rows) v = *(const uint4 *)(base + (long long)k * ld + gr);
        }
      }
      r[i] = v;
    }
  }
  __device__ __forceinline__ void store(bf16_t *S) const {
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int c = threadIdx.x + NTHR * i;
      if (NCH % NTHR == 0 || c < NCH) *(uint4 *)(S + (c / CPR) * PITCH + (c % CPR) * 8) = r[i];
    }
  }
  // Per-lane element offset of the fragment of MFMA tile row block r0 (k step 0); add frag_step(kk).
  static __device__ __forceinline__ int frag_base(int r0, int lane) {
    if constexpr (LAYOUT == 0) return (r0 + (lane & 31)) * PITCH + (lane >> 5) * 8;
    else {
      const int grp = lane >> 4, j = lane & 15;          // 16-lane groups: (k half, row half)
      return (8 * (grp >> 1) + (j >> 2)) * PITCH + r0 + 16 * (grp & 1) + 4 * (j & 3);
    }
  }
  static __device__ __forceinline__ bf16x8_t frag(const bf16_t *S, int off, int kk) {
    if constexpr (LAYOUT == 0) return *(const bf16x8_t *)(S + off + kk * 16);
    else {
      // lane j of a 16-lane group receives column j of the 4(k) x 16(row) patch the group addresses
      const bf16_t *p = S + off + kk * 16 * PITCH;
      const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)p);
      const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)(p + 4 * PITCH));
      typedef __attribute__((ext_vector_type(8))) short s16x8_t;
      const s16x8_t v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      return __builtin_bit_cast(bf16x8_t, v);
    }
  }
};

constexpr int GROUP_M = 8;   // m tiles per swizzle group (L2 reuse of the B tiles)

template <int BM, int BN, int WGM, int WGN, int LA, int LB>
__global__ __launch_bounds__(64 * WGM * WGN) void gemm_bf16_kernel(const GemmParams p) {
  constexpr int NTHR = 64 * WGM * WGN;
  constexpr int WTM = BM / WGM, WTN = BN / WGN;  // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;    // 32x32 MFMA tiles per wave
  using SA = TileStage<BM, LA, NTHR>;
  using SB = TileStage<BN, LB, NTHR>;
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t *As = (bf16_t *)smem_raw;               // [2] stages of A
  bf16_t *Bs = As + 2 * SA::ELEMS;               // [2] stages of B

  // block -> tile.  Consecutive block ids go to different XCDs (8 of them, one L2 each), so each
  // XCD takes a contiguous chunk of the tile list; inside it tiles run over GROUP_M m tiles at
  // a time so that the tiles resident on one XCD share A and B panels.
  const int total_mt = p.mt_start[p.n_mg], total_nt = p.nt_start[p.n_ns];
  const int total = total_mt * total_nt;
  int v;
  {
    const int per = total >> 3, rem = total & 7, xcd = blockIdx.x & 7, idx = blockIdx.x >> 3;
    v = xcd < rem ? xcd * (per + 1) + idx : rem * (per + 1) + (xcd - rem) * per + idx;
  }
  const int grp_sz = GROUP_M * total_nt;
  const int first_m = (v / grp_sz) * GROUP_M;
  const int gm = min(total_mt - first_m, GROUP_M);
  const int mt_g = first_m + (v % grp_sz) % gm, nt_g = (v % grp_sz) / gm;
  int g = 0, s = 0;
  while (g + 1 < p.n_mg && mt_g >= p.mt_start[g + 1]) ++g;
  while (s + 1 < p.n_ns && nt_g >= p.nt_start[s + 1]) ++s;
  const GemmMGroup &G = p.mg[g];
  const GemmNSeg &S = p.ns[s];
  const int m0 = (mt_g - p.mt_start[g]) * BM, n0 = (nt_g - p.nt_start[s]) * BN;
  const int M = G.M, N = S.N, K = p.K;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave / WGN, wn = wave % WGN;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (K + BK - 1) / BK;
  const int n_it = nk * G.npass;
  SA sa;
  SB sb;
  auto issue = [&](int it) {
    const int pass = it / nk, kt = it - pass * nk;
    sa.load(G.a[pass == 1 ? 1 : 0], p.lda, m0, M, kt * BK, K);
    sb.load(S.b[pass == 2 ? 1 : 0], p.ldb, n0, N, kt * BK, K);
  };
  int aoff[TM], boff[TN];
#pragma unroll
  for (int i = 0; i < TM; ++i) aoff[i] = SA::frag_base(wm * WTM + i * 32, lane);
#pragma unroll
  for (int j = 0; j < TN; ++j) boff[j] = SB::frag_base(wn * WTN + j * 32, lane);

  issue(0);
  sa.store(As);
  sb.store(Bs);
  __syncthreads();

  bf16x8_t af[2][TM], bfr[2][TN];                 // fragments double-buffered over the k steps
  for (int it = 0; it < n_it; ++it) {
    const int cur = it & 1;
    if (it + 1 < n_it) issue(it + 1);             // global loads fly during the MFMA phase
    const bf16_t *Ac = As + cur * SA::ELEMS, *Bc = Bs + cur * SB::ELEMS;
#pragma unroll
    for (int i = 0; i < TM; ++i) af[0][i] = SA::frag(Ac, aoff[i], 0);
#pragma unroll
    for (int j = 0; j < TN; ++j) bfr[0][j] = SB::frag(Bc, boff[j], 0);
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      // the LDS reads of step kk+1 are issued ahead of the MFMAs of step kk; the fences keep the
      // compiler from sinking them back next to their uses
      if (kk + 1 < BK / 16) {
#pragma unroll
        for (int i = 0; i < TM; ++i) af[(kk + 1) & 1][i] = SA::frag(Ac, aoff[i], kk + 1);
#pragma unroll
        for (int j = 0; j < TN; ++j) bfr[(kk + 1) & 1][j] = SB::frag(Bc, boff[j], kk + 1);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[kk & 1][i], bfr[kk & 1][j], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
    }
    if (it + 1 < n_it) {
      sa.store(As + (cur ^ 1) * SA::ELEMS);
      sb.store(Bs + (cur ^ 1) * SB::ELEMS);
    }
    __syncthreads();
  }

  // epilogue: accumulator register r of a 32x32 tile holds row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
  const int rk = p.resid_kind, obf = p.out_bf16;
  const long long ldc = p.ldc, ldr = p.ldr;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn * WTN + j * 32 + (lane & 31);
      const int rbase = m0 + wm * WTM + i * 32 + 4 * (lane >> 5);
      if (col >= N) continue;
      const long long cc = S.c_col + col;
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
  for (int s = 0; s < p.n_ns; ++s) { p.nt_start[s] = nt; nt += cdiv(p.ns[s].N, BN); }
  p.nt_start[p.n_ns] = nt;
  return mt * nt;
}

template <int BM, int BN, int WGM, int WGN, int LA, int LB>
hipError_t launch_t(GemmParams &p, hipStream_t stream) {
  const int tiles = count_tiles<BM, BN>(p);
  if (tiles == 0) return hipSuccess;
  constexpr int NTHR = 64 * WGM * WGN;
  constexpr size_t lds = (size_t)2 * (TileStage<BM, LA, NTHR>::ELEMS + TileStage<BN, LB, NTHR>::ELEMS) * sizeof(bf16_t);
  static_assert(lds <= 160 * 1024, "LDS budget of a gfx950 CU");
  static bool attr_done = false;   // per instantiation; setting it twice is harmless
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void *)gemm_bf16_kernel<BM, BN, WGM, WGN, LA, LB>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, WGM, WGN, LA, LB>), dim3((unsigned)tiles), dim3(NTHR), lds, stream, p);
  return hipGetLastError();
}

bool aligned16(const void *q) { return ((uintptr_t)q & 15) == 0; }

int g_force_tile = -1;

template <int LA, int LB>
hipError_t launch_layout(GemmParams &p, hipStream_t stream) {
  int tile = g_force_tile;
  if (tile < 0) {
    // 256x256 tiles (8 waves) halve the LDS and L2 traffic per flop; use them once they still
    // give every CU at least two tiles, else 128x128 tiles (4 waves, two blocks per CU).
    GemmParams q = p;
    tile = count_tiles<256, 256>(q) >= 512 ? 3 : 0;
  }
  switch (tile) {
    case 3: return launch_t<256, 256, 2, 4, LA, LB>(p, stream);
    case 4: return launch_t<256, 128, 4, 2, LA, LB>(p, stream);
    default: return launch_t<128, 128, 2, 2, LA, LB>(p, stream);
  }
}

}  // namespace

// development hook: pin the tile configuration (-1 = automatic)
void gemm_force_tile(int id) { g_force_tile = id; }

hipError_t gemm_launch(int LA, int LB, GemmParams &p, hipStream_t stream, const char **why) {
  *why = nullptr;
  if (p.n_mg < 1 || p.n_mg > 3 || p.n_ns < 1 || p.n_ns > 3) { *why = "gemm: group count"; return hipErrorInvalidValue; }
  if (p.K <= 0) { *why = "gemm: K <= 0"; return hipErrorInvalidValue; }
  if ((LA == 0 || LB == 0) && p.K % BK) { *why = "gemm: K of a k-contiguous operand must be a multiple of 64"; return hipErrorInvalidValue; }
  if (p.lda % 8 || p.ldb % 8) { *why = "gemm: leading dimension not a multiple of 8"; return hipErrorInvalidValue; }
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
  if (LA == 0 && LB == 0) return launch_layout<0, 0>(p, stream);
  if (LA == 0 && LB == 1) return launch_layout<0, 1>(p, stream);
  if (LA == 1 && LB == 1) return launch_layout<1, 1>(p, stream);
  *why = "gemm: unsupported layout";
  return hipErrorInvalidValue;
}
