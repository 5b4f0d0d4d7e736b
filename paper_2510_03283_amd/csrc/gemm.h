// Grouped bf16 MFMA GEMM used by every dense contraction of the iteration.
#pragma once
#include "common.h"

// C[m, n] = sum_k A[m, k] * B[n, k]  (+ residual), over up to three row groups that share B and
// up to three column segments that share A.  Row groups let inference rows (one bf16 pass) and
// fine-tune rows (two- or three-pass split operands) ride in one launch; column segments let
// several weight matrices with separate base pointers (Wq|Wk|Wv, Wg|Wu) ride in one launch.
//
// Operand layouts (element type bf16):
//   LA = 0: A is [M, K] row-major (k contiguous).   LA = 1: A is [K, M] row-major (m contiguous).
//   LB = 0: B is [N, K] row-major (k contiguous).   LB = 1: B is [K, N] row-major (n contiguous).
// Requirements checked by gemm_launch: K % 64 == 0 for a k-contiguous operand; M % 8 == 0
// (N % 8 == 0) for an m- (n-) contiguous operand; all leading dimensions and column offsets
// multiples of 8 elements; pointers 16-byte aligned.
struct GemmMGroup {
  const bf16_t *a[2];   // [0] = hi (or only) operand, [1] = lo term (passes 2..)
  void *c;              // first output row of the group
  const void *resid;    // first residual row of the group (may be null)
  int M;                // rows in the group
  int npass;            // 1: A0*B0   2: + A1*B0   3: + A0*B1
  // SwiGLU mode only: c receives hm = silu(G) * U as bf16 [M, F]; c_lo (nullable) its second bf16
  // term; c_gu (nullable) G and U as bf16 [M, 2F] (G in columns [0,F), U in [F,2F)).
  void *c_lo;
  void *c_gu;
  // Rotary mode (NT form, four-wave kernel only - ask gemm_uses_four_wave first; head dimension 128): 1 = the rows
  // of this group are not written to c; every column segment writes its part as two bf16 terms [M, N] (row stride
  // N) into its rope_hi / rope_lo, rotated by the group's angle table where the segment says so.
  int rope;
};
struct GemmNSeg {
  const bf16_t *b[2];   // [0] = hi (or only) operand, [1] = lo term (pass 3)
  int N;                // columns in the segment
  int c_col;            // first output column of the segment
  // rotary mode (row groups with rope = 1): outputs of this segment and whether its heads are rotated (Q, K) or
  // only split into two terms (V)
  void *rope_hi, *rope_lo;
  int rope_rot;
};
struct GemmParams {
  GemmMGroup mg[3];
  GemmNSeg ns[3];
  int n_mg, n_ns;
  int K;
  long long lda, ldb, ldc, ldr;
  int out_bf16;     // 0: C is fp32, 1: C is bf16
  int resid_kind;   // 0 none, 1 fp32, 2 bf16 ; C = acc + resid
  // K segments (optional, n_kseg > 1; needs n_ns == 1 and one pass): the k range is a concatenation
  // and segment s (k in [kseg_start[s], kseg_start[s+1]), boundaries multiples of 64) takes its B
  // rows from kseg_b[s] instead of ns[0].b[0] - several weight matrices stacked along the reduction
  // (dX = dQ Wq + dK Wk + dV Wv as one product).
  int n_kseg;
  const bf16_t *kseg_b[3];
  int kseg_start[4];
  // SwiGLU mode (NT form only): ns[0] = gate weights, ns[1] = up weights, both [F, K]; every wave
  // multiplies 32 gate columns and the 32 up columns of the same hidden units, and the epilogue
  // writes silu(G) * U instead of G and U (ldc = F).
  int swiglu;
  int k_splits;     // > 1: grid.y slices of the k range; slice z writes fp32 partial sums at C + z * c_split_stride
  long long c_split_stride;   // elements
  int mt_start[4];  // filled by gemm_launch
  int nt_start[4];
  int tile_m, tile_n;   // filled by gemm_launch: the block tile its cost model chose
  // SwiGLU backward mode (NN form, four-wave kernel only - ask gemm_uses_four_wave first): the product is dHm [M, N = F];
  // instead of it the epilogue writes dG | dU as bf16 [M, 2F] into c (ldc = 2F) from G | U of the forward, bf16 [M, 2F]
  // in c_gu (read only): dG = dHm U s (1 + G (1 - s)), dU = dHm G s, s = sigmoid(G).
  int swiglu_bwd;
  const float *rope_cs;   // rotary mode: (cos, sin) of row r of the rope group and pair index i at rope_cs[2 (64 r + i)]
  int force_w4;     // 1: the 256x256 four-wave kernel whatever the cost model says (rejected if the problem does not fit it)
};

// Number of k slices worth using for a single-group, single-segment problem (1 = none): small
// outputs with a long reduction leave most CUs idle otherwise.  Priced with the launcher's tile
// cost model plus the traffic of writing and summing the partial results.
int gemm_suggest_k_splits(int M, int N, int K);

// Whether gemm_launch would run this problem on the four-wave kernel (its cost model picks the 256x256 tile, or
// force_w4 is set, and the problem fits the kernel).  Forms that only that kernel has are launched after asking.
bool gemm_uses_four_wave(int LA, int LB, const GemmParams &p);

// Returns hipSuccess or the launch error; a non-null *why is set on a rejected shape.
hipError_t gemm_launch(int LA, int LB, GemmParams &p, hipStream_t stream, const char **why);
