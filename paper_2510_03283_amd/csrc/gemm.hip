// bf16 MFMA GEMM for gfx950: 256 threads (2x2 waves), 32x32x16 MFMA tiles, LDS double buffer.
#include "gemm.h"

namespace {

constexpr int BK = 64;          // k extent of an LDS tile
constexpr int LDK = BK + 8;     // LDS row pitch in elements: 144 B keeps 16-byte reads conflict-free

// Global -> register -> LDS staging of a ROWS x BK operand tile.
// LAYOUT 0: memory is [row][k]; each thread moves 16-byte chunks (8 k of one row).
// LAYOUT 1: memory is [k][row]; each thread loads a 4(k) x 8(row) block, transposes it in
//           registers and writes 8 rows x 4 k, so that LDS always holds [row][k].
template <int ROWS, int LAYOUT>
struct TileStage {
  static constexpr int NV = ROWS / 32;
  uint4 r[NV];

  __device__ __forceinline__ void load(const bf16_t *base, long long ld, int row0, int rows, int k0, int K) {
    const int tid = threadIdx.x;
    if constexpr (LAYOUT == 0) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = tid + 256 * i;
        const int row = c >> 3, kc = c & 7;
        const int gr = row0 + row;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (gr < rows) v = *(const uint4 *)(base + (long long)gr * ld + k0 + kc * 8);
        r[i] = v;
      }
    } else {
      static_assert(LAYOUT == 0 || ROWS % 128 == 0, "transposing stage needs ROWS % 128 == 0");
#pragma unroll
      for (int i = 0; i < ROWS / 128; ++i) {
        const int c = tid + 256 * i;
        const int mblk = c % (ROWS / 8), kblk = c / (ROWS / 8);
        const int gr = row0 + 8 * mblk;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          const int k = k0 + 4 * kblk + j;
          uint4 v = make_uint4(0, 0, 0, 0);
          if (gr < rows && k < K) v = *(const uint4 *)(base + (long long)k * ld + gr);
          r[4 * i + j] = v;
        }
      }
    }
  }

  __device__ __forceinline__ void store(bf16_t *S) const {
    const int tid = threadIdx.x;
    if constexpr (LAYOUT == 0) {
#pragma unroll
      for (int i = 0; i < NV; ++i) {
        const int c = tid + 256 * i;
        const int row = c >> 3, kc = c & 7;
        *(uint4 *)(S + row * LDK + kc * 8) = r[i];
      }
    } else {
#pragma unroll
      for (int i = 0; i < ROWS / 128; ++i) {
        const int c = tid + 256 * i;
        const int mblk = c % (ROWS / 8), kblk = c / (ROWS / 8);
        uint32_t d[4][4];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          d[j][0] = r[4 * i + j].x; d[j][1] = r[4 * i + j].y; d[j][2] = r[4 * i + j].z; d[j][3] = r[4 * i + j].w;
        }
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
          *(uint2 *)(S + (8 * mblk + m) * LDK + 4 * kblk) = make_uint2(w0, w1);
        }
      }
    }
  }
};

template <int BM, int BN, int LA, int LB>
__global__ __launch_bounds__(256) void gemm_bf16_kernel(const GemmParams p) {
  constexpr int WTM = BM / 2, WTN = BN / 2;      // wave tile
  constexpr int TM = WTM / 32, TN = WTN / 32;    // 32x32 MFMA tiles per wave
  extern __shared__ __align__(16) unsigned char smem_raw[];
  bf16_t *As = (bf16_t *)smem_raw;               // [2][BM][LDK]
  bf16_t *Bs = As + 2 * BM * LDK;                // [2][BN][LDK]

  // tile -> (row group, m tile, column segment, n tile); n fastest
  const int total_nt = p.nt_start[p.n_ns];
  const int mt_g = blockIdx.x / total_nt, nt_g = blockIdx.x % total_nt;
  int g = 0, s = 0;
  while (g + 1 < p.n_mg && mt_g >= p.mt_start[g + 1]) ++g;
  while (s + 1 < p.n_ns && nt_g >= p.nt_start[s + 1]) ++s;
  const GemmMGroup &G = p.mg[g];
  const GemmNSeg &S = p.ns[s];
  const int m0 = (mt_g - p.mt_start[g]) * BM, n0 = (nt_g - p.nt_start[s]) * BN;
  const int M = G.M, N = S.N, K = p.K;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int wm = wave >> 1, wn = wave & 1;

  f32x16_t acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.f;

  const int nk = (K + BK - 1) / BK;
  const int n_it = nk * G.npass;
  TileStage<BM, LA> sa;
  TileStage<BN, LB> sb;

  auto issue = [&](int it) {
    const int pass = it / nk, kt = it - pass * nk;
    const bf16_t *a = G.a[pass == 1 ? 1 : 0];
    const bf16_t *b = S.b[pass == 2 ? 1 : 0];
    sa.load(a, p.lda, m0, M, kt * BK, K);
    sb.load(b, p.ldb, n0, N, kt * BK, K);
  };

  issue(0);
  sa.store(As);
  sb.store(Bs);
  __syncthreads();

  for (int it = 0; it < n_it; ++it) {
    const int cur = it & 1;
    if (it + 1 < n_it) issue(it + 1);
    const bf16_t *Ac = As + cur * BM * LDK + (wm * WTM + (lane & 31)) * LDK + (lane >> 5) * 8;
    const bf16_t *Bc = Bs + cur * BN * LDK + (wn * WTN + (lane & 31)) * LDK + (lane >> 5) * 8;
#pragma unroll
    for (int kk = 0; kk < BK / 16; ++kk) {
      bf16x8_t af[TM], bfr[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) af[i] = *(const bf16x8_t *)(Ac + i * 32 * LDK + kk * 16);
#pragma unroll
      for (int j = 0; j < TN; ++j) bfr[j] = *(const bf16x8_t *)(Bc + j * 32 * LDK + kk * 16);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(af[i], bfr[j], acc[i][j], 0, 0, 0);
    }
    if (it + 1 < n_it) {
      sa.store(As + (cur ^ 1) * BM * LDK);
      sb.store(Bs + (cur ^ 1) * BN * LDK);
    }
    __syncthreads();
  }

  // epilogue: accumulator register r of a 32x32 tile holds row 8*(r/4) + 4*(lane/32) + r%4, column lane%32
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int col = n0 + wn * WTN + j * 32 + (lane & 31);
      if (col >= N) continue;
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int row = m0 + wm * WTM + i * 32 + 8 * (r >> 2) + 4 * (lane >> 5) + (r & 3);
        if (row >= M) continue;
        float v = acc[i][j][r];
        if (p.resid_kind == 1) v += ((const float *)G.resid)[(long long)row * p.ldr + S.c_col + col];
        else if (p.resid_kind == 2) v += bf2f(((const bf16_t *)G.resid)[(long long)row * p.ldr + S.c_col + col]);
        const long long o = (long long)row * p.ldc + S.c_col + col;
        if (p.out_bf16) ((bf16_t *)G.c)[o] = f2bf(v);
        else ((float *)G.c)[o] = v;
      }
    }
  }
}

template <int BM, int BN, int LA, int LB>
hipError_t launch_t(GemmParams &p, hipStream_t stream) {
  int mt = 0, nt = 0;
  for (int g = 0; g < p.n_mg; ++g) { p.mt_start[g] = mt; mt += cdiv(p.mg[g].M, BM); }
  p.mt_start[p.n_mg] = mt;
  for (int s = 0; s < p.n_ns; ++s) { p.nt_start[s] = nt; nt += cdiv(p.ns[s].N, BN); }
  p.nt_start[p.n_ns] = nt;
  if (mt == 0 || nt == 0) return hipSuccess;
  constexpr size_t lds = (size_t)2 * (BM + BN) * LDK * sizeof(bf16_t);
  static bool attr_done = false;   // per instantiation; setting it twice is harmless
  if (!attr_done) {
    hipError_t e = hipFuncSetAttribute((const void *)gemm_bf16_kernel<BM, BN, LA, LB>,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    attr_done = true;
  }
  hipLaunchKernelGGL((gemm_bf16_kernel<BM, BN, LA, LB>), dim3((unsigned)(mt * nt)), dim3(256), lds, stream, p);
  return hipGetLastError();
}

bool aligned16(const void *q) { return ((uintptr_t)q & 15) == 0; }

}  // namespace

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
  if (LA == 0 && LB == 0) return launch_t<128, 128, 0, 0>(p, stream);
  if (LA == 0 && LB == 1) return launch_t<128, 128, 0, 1>(p, stream);
  if (LA == 1 && LB == 1) return launch_t<128, 128, 1, 1>(p, stream);
  *why = "gemm: unsupported layout";
  return hipErrorInvalidValue;
}
