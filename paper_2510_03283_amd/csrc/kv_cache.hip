// Paged KV cache, layout [blocks, Hkv, B, hd] for K and V each: scatter by slot, gather by block table.
// Element offset of (slot, kv head, e) = ((slot / B) * Hkv + kvh) * B * hd + (slot % B) * hd + e, in 64 bits.
#include "kernels.h"

namespace {

// One block per new row; payload copied in 4-byte words (ELT = bytes per element, row = Hkv*hd elements).
template <int ELT>
__global__ __launch_bounds__(256) void kv_append_kernel(unsigned char *ck, unsigned char *cv, long long num_slots,
                                                        int B, int Hkv, int hd, const unsigned char *kn,
                                                        const unsigned char *vn, const int32_t *slot_mapping) {
  const int r = blockIdx.x;
  const long long slot = slot_mapping[r];
  if (slot < 0 || slot >= num_slots) return;
  const long long base = (slot / B) * (long long)Hkv * B * hd + (slot % B) * (long long)hd;
  const int wph = hd * ELT / 4;                 // 4-byte words per head row
  const int nw = Hkv * wph;
  const uint32_t *ks = (const uint32_t *)(kn + (size_t)r * Hkv * hd * ELT);
  const uint32_t *vs = (const uint32_t *)(vn + (size_t)r * Hkv * hd * ELT);
  for (int w = threadIdx.x; w < nw; w += 256) {
    const int kh = w / wph, e = w - kh * wph;
    const long long o = (base + (long long)kh * B * hd) * ELT / 4 + e;
    ((uint32_t *)ck)[o] = ks[w];
    ((uint32_t *)cv)[o] = vs[w];
  }
}

// One block per context position.
template <int ELT>
__global__ __launch_bounds__(256) void kv_gather_kernel(const unsigned char *ck, const unsigned char *cv,
                                                        long long num_blocks, int B, int Hkv, int hd,
                                                        const int32_t *block_table, unsigned char *ko,
                                                        unsigned char *vo, long long *slots_out) {
  const int p = blockIdx.x;
  const long long blk = block_table[p / B];
  const long long slot = blk * B + p % B;
  if (slots_out && threadIdx.x == 0) slots_out[p] = slot;
  const int wph = hd * ELT / 4;
  const int nw = Hkv * wph;
  uint32_t *kd = (uint32_t *)(ko + (size_t)p * Hkv * hd * ELT);
  uint32_t *vd = (uint32_t *)(vo + (size_t)p * Hkv * hd * ELT);
  const bool ok = blk >= 0 && blk < num_blocks;   // a bad table entry yields zeros, never a wild read
  const long long base = blk * (long long)Hkv * B * hd + (p % B) * (long long)hd;
  for (int w = threadIdx.x; w < nw; w += 256) {
    const int kh = w / wph, e = w - kh * wph;
    const long long o = (base + (long long)kh * B * hd) * ELT / 4 + e;
    kd[w] = ok ? ((const uint32_t *)ck)[o] : 0u;
    vd[w] = ok ? ((const uint32_t *)cv)[o] : 0u;
  }
}

}  // namespace

hipError_t launch_kv_append(void *cache_k, void *cache_v, bool bf16, long long num_slots, int block_size, int Hkv,
                            int hd, const void *k_new, const void *v_new, const int32_t *slot_mapping, int n,
                            hipStream_t st) {
  if (n <= 0) return hipSuccess;
  if (bf16)
    hipLaunchKernelGGL((kv_append_kernel<2>), dim3(n), dim3(256), 0, st, (unsigned char *)cache_k, (unsigned char *)cache_v, num_slots, block_size, Hkv, hd, (const unsigned char *)k_new, (const unsigned char *)v_new, slot_mapping);
  else
    hipLaunchKernelGGL((kv_append_kernel<4>), dim3(n), dim3(256), 0, st, (unsigned char *)cache_k, (unsigned char *)cache_v, num_slots, block_size, Hkv, hd, (const unsigned char *)k_new, (const unsigned char *)v_new, slot_mapping);
  return hipGetLastError();
}

hipError_t launch_kv_gather(const void *cache_k, const void *cache_v, bool bf16, long long num_blocks, int block_size,
                            int Hkv, int hd, const int32_t *block_table, int ctx_len, void *k_out, void *v_out,
                            long long *slots_out, hipStream_t st) {
  if (ctx_len <= 0) return hipSuccess;
  if (bf16)
    hipLaunchKernelGGL((kv_gather_kernel<2>), dim3(ctx_len), dim3(256), 0, st, (const unsigned char *)cache_k, (const unsigned char *)cache_v, num_blocks, block_size, Hkv, hd, block_table, (unsigned char *)k_out, (unsigned char *)v_out, slots_out);
  else
    hipLaunchKernelGGL((kv_gather_kernel<4>), dim3(ctx_len), dim3(256), 0, st, (const unsigned char *)cache_k, (const unsigned char *)cache_v, num_blocks, block_size, Hkv, hd, block_table, (unsigned char *)k_out, (unsigned char *)v_out, slots_out);
  return hipGetLastError();
}
