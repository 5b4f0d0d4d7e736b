// The two small pieces that close the loop around an iteration: the greedy next token of
// inference rows from their logits (what the serving loop samples and checks for end of sequence)
// and the AdamW update that turns an iteration's gradients into the next iteration's weights.
#include "kernels.h"

namespace {

// One block per row: arg max over V fp32 logits, lowest index on ties.
__global__ __launch_bounds__(256) void argmax_rows_kernel(const float *__restrict__ logits, int V, int32_t *__restrict__ out) {
  const float *row = logits + (size_t)blockIdx.x * V;
  float best = -INFINITY;
  int bi = 0x7fffffff;
  for (int j = threadIdx.x; j < V; j += 256) {
    const float v = row[j];
    if (v > best || (v == best && j < bi)) { best = v; bi = j; }
  }
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) {
    const float ov = __shfl_xor(best, o, 64);
    const int oi = __shfl_xor(bi, o, 64);
    if (ov > best || (ov == best && oi < bi)) { best = ov; bi = oi; }
  }
  __shared__ float sv[4];
  __shared__ int si[4];
  const int w = threadIdx.x >> 6;
  if ((threadIdx.x & 63) == 0) { sv[w] = best; si[w] = bi; }
  __syncthreads();
  if (threadIdx.x == 0) {
    for (int k = 1; k < 4; ++k)
      if (sv[k] > best || (sv[k] == best && si[k] < bi)) { best = sv[k]; bi = si[k]; }
    out[blockIdx.x] = bi == 0x7fffffff ? 0 : bi;       // a row of NaNs / -inf yields 0
  }
}

// AdamW, decoupled weight decay; c1 = 1/(1-b1^t), c2 = 1/(1-b2^t) come from the host in fp64 -> fp32.
struct AdamW {
  float lr, b1, b2, eps, wd, c1, c2;
  __device__ __forceinline__ float step(float g, float &m, float &v, float p) const {
    m = b1 * m + (1.f - b1) * g;
    v = b2 * v + (1.f - b2) * g * g;
    return p - lr * ((m * c1) / (sqrtf(v * c2) + eps) + wd * p);
  }
};

// Four elements per thread with 16-byte accesses (HBM-bound: 26-30 bytes per element); the last
// n % 4 elements are done one by one by the first threads.
template <bool PBF16>
__global__ __launch_bounds__(256) void adamw_kernel(void *__restrict__ param, float *__restrict__ master, const float *__restrict__ grad,
                                                    float *__restrict__ m, float *__restrict__ v, size_t n, const AdamW a) {
  const size_t n4 = n / 4, stride = (size_t)gridDim.x * 256;
  for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n4; i += stride) {
    const float4 g = ((const float4 *)grad)[i];
    float4 mi = ((float4 *)m)[i], vi = ((float4 *)v)[i], p;
    if (master) p = ((const float4 *)master)[i];
    else if constexpr (PBF16) {
      const uint2 r = ((const uint2 *)param)[i];
      p = make_float4(__uint_as_float(r.x << 16), __uint_as_float(r.x & 0xffff0000u), __uint_as_float(r.y << 16), __uint_as_float(r.y & 0xffff0000u));
    } else p = ((const float4 *)param)[i];
    p.x = a.step(g.x, mi.x, vi.x, p.x);
    p.y = a.step(g.y, mi.y, vi.y, p.y);
    p.z = a.step(g.z, mi.z, vi.z, p.z);
    p.w = a.step(g.w, mi.w, vi.w, p.w);
    ((float4 *)m)[i] = mi;
    ((float4 *)v)[i] = vi;
    if (master) ((float4 *)master)[i] = p;
    if constexpr (PBF16) ((uint2 *)param)[i] = make_uint2(pack2(f2bf(p.x), f2bf(p.y)), pack2(f2bf(p.z), f2bf(p.w)));
    else ((float4 *)param)[i] = p;
  }
  const size_t i = n4 * 4 + (size_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) {
    float mi = m[i], vi = v[i];
    const float p = a.step(grad[i], mi, vi, master ? master[i] : ld_io<PBF16>(param, i));
    m[i] = mi;
    v[i] = vi;
    if (master) master[i] = p;
    st_io<PBF16>(param, i, p);
  }
}

}  // namespace

hipError_t launch_argmax_rows(const float *logits, int rows, int V, int32_t *out, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  hipLaunchKernelGGL(argmax_rows_kernel, dim3(rows), dim3(256), 0, st, logits, V, out);
  return hipGetLastError();
}

hipError_t launch_adamw(void *param, bool param_bf16, float *master, const float *grad, float *m, float *v, size_t n, float lr,
                        float b1, float b2, float eps, float wd, float c1, float c2, hipStream_t st) {
  if (n == 0) return hipSuccess;
  const size_t want = (n / 4 + 255) / 256 + 1;
  const unsigned blocks = (unsigned)(want < 8192 ? want : 8192);
  const AdamW a{lr, b1, b2, eps, wd, c1, c2};
  const uintptr_t al = (uintptr_t)param | (uintptr_t)master | (uintptr_t)grad | (uintptr_t)m | (uintptr_t)v;
  if (al & 15) return hipErrorInvalidValue;       // 16-byte accesses
  if (param_bf16) hipLaunchKernelGGL(adamw_kernel<true>, dim3(blocks), dim3(256), 0, st, param, master, grad, m, v, n, a);
  else hipLaunchKernelGGL(adamw_kernel<false>, dim3(blocks), dim3(256), 0, st, param, master, grad, m, v, n, a);
  return hipGetLastError();
}
