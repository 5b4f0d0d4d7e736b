// Small helpers of the adapter (LoRA) variant: packing the caller's rank-r adapter matrices into
// zero-padded bf16 operands the GEMM accepts (rank padded to 64; the three q/k/v adapters stacked
// into one [3*64, d] A matrix and one block-diagonal [(Hq+2Hkv)*hd, 3*64] B matrix), scaling the
// low-rank activations, and cutting the adapter gradients back out of the padded products.
#include "kernels.h"

namespace {

struct PackSrc {
  const void *p;     // [rows, cols] row-major, fp32 or bf16
  int rows, cols;
  int r0, c0;        // placement of element (0, 0) in the destination
};

// dst[dst_rows, dst_cols] (hi, optional lo) = zeros, except the windows covered by up to 3 sources.
template <bool BF16>
__global__ __launch_bounds__(256) void lora_pack_kernel(PackSrc s0, PackSrc s1, PackSrc s2, int n_src, int dst_rows, int dst_cols, float scale,
                                                        bf16_t *__restrict__ hi, bf16_t *__restrict__ lo) {
  const size_t n = (size_t)dst_rows * dst_cols, stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
    const int r = (int)(i / dst_cols), c = (int)(i % dst_cols);
    float v = 0.f;
    const PackSrc *ss[3] = {&s0, &s1, &s2};
#pragma unroll
    for (int k = 0; k < 3; ++k)
      if (k < n_src) {
        const int rr = r - ss[k]->r0, cc = c - ss[k]->c0;
        if (rr >= 0 && rr < ss[k]->rows && cc >= 0 && cc < ss[k]->cols) v = ld_io<BF16>(ss[k]->p, (size_t)rr * ss[k]->cols + cc);
      }
    bf16_t h, l;
    split_bf(v * scale, h, l);
    hi[i] = h;
    if (lo) lo[i] = l;
  }
}

__global__ __launch_bounds__(256) void scale_split_kernel(const float *__restrict__ src, size_t n, float scale,
                                                          bf16_t *__restrict__ hi, bf16_t *__restrict__ lo) {
  const size_t stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
    bf16_t h, l;
    split_bf(src[i] * scale, h, l);
    hi[i] = h;
    if (lo) lo[i] = l;
  }
}

// dst[rows, cols] (+)= src[(r0 + i) * src_ld + c0 + j]
__global__ __launch_bounds__(256) void extract_kernel(const float *__restrict__ src, int src_ld, int r0, int c0, int rows, int cols,
                                                      float scale, float *__restrict__ dst, int accumulate) {
  const size_t n = (size_t)rows * cols, stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += stride) {
    const int r = (int)(i / cols), c = (int)(i % cols);
    const float v = scale * src[(size_t)(r0 + r) * src_ld + c0 + c];
    dst[i] = accumulate ? dst[i] + v : v;
  }
}

unsigned grid_for(size_t n) { return (unsigned)((n + 255) / 256 < 2048 ? (n + 255) / 256 : 2048); }

}  // namespace

hipError_t launch_lora_pack(const void *const *src, const int *rows, const int *cols, const int *r0, const int *c0, int n_src,
                            bool src_bf16, int dst_rows, int dst_cols, float scale, bf16_t *hi, bf16_t *lo, hipStream_t st) {
  if (n_src < 1 || n_src > 3 || dst_rows <= 0 || dst_cols <= 0) return hipErrorInvalidValue;
  PackSrc s[3] = {};
  for (int k = 0; k < n_src; ++k) {
    if (!src[k] || rows[k] <= 0 || cols[k] <= 0 || r0[k] < 0 || c0[k] < 0 || r0[k] + rows[k] > dst_rows || c0[k] + cols[k] > dst_cols) return hipErrorInvalidValue;
    s[k] = PackSrc{src[k], rows[k], cols[k], r0[k], c0[k]};
  }
  const size_t n = (size_t)dst_rows * dst_cols;
  if (src_bf16) hipLaunchKernelGGL(lora_pack_kernel<true>, dim3(grid_for(n)), dim3(256), 0, st, s[0], s[1], s[2], n_src, dst_rows, dst_cols, scale, hi, lo);
  else hipLaunchKernelGGL(lora_pack_kernel<false>, dim3(grid_for(n)), dim3(256), 0, st, s[0], s[1], s[2], n_src, dst_rows, dst_cols, scale, hi, lo);
  return hipGetLastError();
}

hipError_t launch_scale_split(const float *src, size_t n, float scale, bf16_t *hi, bf16_t *lo, hipStream_t st) {
  if (n == 0) return hipSuccess;
  hipLaunchKernelGGL(scale_split_kernel, dim3(grid_for(n)), dim3(256), 0, st, src, n, scale, hi, lo);
  return hipGetLastError();
}

hipError_t launch_extract(const float *src, int src_ld, int r0, int c0, int rows, int cols, float scale, float *dst, int accumulate, hipStream_t st) {
  if (rows <= 0 || cols <= 0) return hipErrorInvalidValue;
  hipLaunchKernelGGL(extract_kernel, dim3(grid_for((size_t)rows * cols)), dim3(256), 0, st, src, src_ld, r0, c0, rows, cols, scale, dst, accumulate);
  return hipGetLastError();
}
