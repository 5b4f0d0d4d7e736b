// Shared device/host helpers of the MI355X hybrid-iteration library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

typedef uint16_t bf16_t;   // raw bfloat16 bits

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;
typedef __attribute__((ext_vector_type(4))) float f32x4_t;

#define MACE_WAVE 64

__device__ __forceinline__ float bf2f(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// fp32 -> bf16, round to nearest even; NaN stays NaN.
__device__ __forceinline__ bf16_t f2bf(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)0x7fc0;
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

// Two-term bf16 representation: f ~= hi + lo with hi = bf16(f), lo = bf16(f - hi).
__device__ __forceinline__ void split_bf(float f, bf16_t &hi, bf16_t &lo) {
  hi = f2bf(f);
  lo = f2bf(f - bf2f(hi));
}

__device__ __forceinline__ uint32_t pack2(bf16_t a, bf16_t b) { return (uint32_t)a | ((uint32_t)b << 16); }

// Two fp32 -> one packed bf16 pair (a in the low half) with the hardware conversion
// (v_cvt_pk_bf16_f32, round to nearest even), and the two-term form of a pair.
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
__device__ __forceinline__ uint32_t cvt_pk_bf16(float a, float b) {
  const f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}
__device__ __forceinline__ void split_pk_bf16(float a, float b, uint32_t &hi, uint32_t &lo) {
  hi = cvt_pk_bf16(a, b);
  lo = cvt_pk_bf16(a - __uint_as_float(hi << 16), b - __uint_as_float(hi & 0xffff0000u));
}

// Element load of an io tensor (fp32 or bf16) as fp32.
template <bool BF16>
__device__ __forceinline__ float ld_io(const void *p, size_t i) {
  if constexpr (BF16) return bf2f(((const bf16_t *)p)[i]);
  else return ((const float *)p)[i];
}
template <bool BF16>
__device__ __forceinline__ void st_io(void *p, size_t i, float v) {
  if constexpr (BF16) ((bf16_t *)p)[i] = f2bf(v);
  else ((float *)p)[i] = v;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
  return v;
}
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, 64));
  return v;
}

// Block-wide sum for blocks of NT threads (NT multiple of 64, <= 1024); red must hold NT/64 floats.
template <int NT>
__device__ __forceinline__ float block_sum(float v, float *red) {
  v = wave_sum(v);
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  __syncthreads();
  if (l == 0) red[w] = v;
  __syncthreads();
  float t = 0.f;
#pragma unroll
  for (int i = 0; i < NT / 64; ++i) t += red[i];
  return t;
}
template <int NT>
__device__ __forceinline__ float block_max(float v, float *red) {
  v = wave_max(v);
  const int w = threadIdx.x >> 6, l = threadIdx.x & 63;
  __syncthreads();
  if (l == 0) red[w] = v;
  __syncthreads();
  float t = red[0];
#pragma unroll
  for (int i = 1; i < NT / 64; ++i) t = fmaxf(t, red[i]);
  return t;
}

// Per-device "done once" flag for launch attributes that HIP keeps per device (dynamic LDS limit):
// one bit per device, set after the attribute call succeeded.  Safe to use from several host
// threads (two threads that race only repeat an idempotent call); a device beyond bit 31 always
// reads false, which costs a repeated call and nothing else.
#include <atomic>
struct DeviceOnce {
  std::atomic<uint32_t> mask{0};
  static int dev() {
    int d = 0;
    (void)hipGetDevice(&d);
    return d;
  }
  bool test() const {
    const int d = dev();
    return d >= 0 && d < 32 && ((mask.load(std::memory_order_acquire) >> d) & 1u);
  }
  void set() {
    const int d = dev();
    if (d >= 0 && d < 32) mask.fetch_or(1u << d, std::memory_order_release);
  }
};

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }
static inline int cdiv(int a, int b) { return (a + b - 1) / b; }
