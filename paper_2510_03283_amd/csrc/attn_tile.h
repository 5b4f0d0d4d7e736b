// LDS tiles of the attention kernels (gfx950): ROWS token rows x HD head-dim elements of one
// head, bf16, in their memory layout [row][HD], filled by direct global->LDS loads.
//
// The same tile serves two kinds of MFMA operand:
//  * frag_k: 8 consecutive head-dim elements of one tile row per lane (reduction over the head
//    dimension), one 16-byte LDS read;
//  * frag_t: for head-dim index r0 + lane%32, the 8 tile rows kk*16 + 8*(lane/32) .. +7
//    (reduction over the tile rows), two transposing 8-byte reads (ds_read_b64_tr_b16);
// so no transposed copy of a tile is ever built.  A wave-wide direct load writes 64 consecutive
// 16-byte chunks, hence tiles are unpadded; the chunk position inside a row is XOR-swizzled
// with a function of the row that keeps BOTH read patterns free of bank conflicts:
// 16 consecutive rows at one logical chunk (frag_k) and 4 consecutive rows x 4 consecutive
// chunks (frag_t) each touch 16 different 16-byte bank groups.
#pragma once
#include "common.h"

namespace attn {

typedef __attribute__((ext_vector_type(4))) short s16x4_t;
typedef __attribute__((ext_vector_type(8))) short s16x8_t;
typedef __attribute__((address_space(3))) s16x4_t lds_s16x4_t;
typedef __attribute__((address_space(3))) void lds_void_t;
typedef __attribute__((address_space(1))) const void gbl_void_t;

static __device__ __align__(16) uint4 zero16 = {0u, 0u, 0u, 0u};   // source of rows beyond the sequence

template <int N>
__device__ __forceinline__ void wait_vmcnt() {   // vmcnt <= N, no wait on the other counters
  __builtin_amdgcn_s_waitcnt((N & 15) | ((N >> 4) << 14) | (7 << 4) | (15 << 8));
}

// swap bits 2 and 3: the MFMA output row held in register r of lane half g is
// 8*(r/4) + 4*g + r%4; reading operand row swap23(i) for MFMA row i makes register r = 8*mm + e
// of half g hold tile row 16*mm + 8*g + e, the order a B operand wants its 8 reduction indices in.
__device__ __forceinline__ int swap23(int i) { return (i & ~12) | ((i & 4) << 1) | ((i & 8) >> 1); }

template <int ROWS, int HD, int NTHR>
struct Tile {
  static constexpr int CPR = HD / 8;                 // 16-byte chunks per row (8 or 16)
  static constexpr int ELEMS = ROWS * HD;
  static constexpr int NCH = ROWS * CPR;
  static constexpr int NI = NCH / NTHR;              // wave-wide loads per wave
  static_assert(HD == 64 || HD == 128, "head dim");
  static_assert(NCH % NTHR == 0, "tile must split evenly over the waves");

  static __device__ __forceinline__ int swz(int row) {
    if constexpr (CPR == 16) return ((row & 3) << 2) | ((row >> 2) & 3);
    else return (((row >> 1) & 1) << 2) | ((row >> 2) & 3);
  }

  // Rows row0 .. row0+ROWS-1 of src (row pitch ld elements; src points at row 0, column 0 of the
  // head); rows >= row_end read zeros.
  static __device__ __forceinline__ void issue(const bf16_t *src, size_t ld, int row0, int row_end, bf16_t *S) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int q = wave + (NTHR / 64) * i;
      const int chunk = q * 64 + lane;
      const int lr = chunk / CPR, c = (chunk % CPR) ^ swz(lr);
      const int gr = row0 + lr;
      const bf16_t *p = gr < row_end ? src + (size_t)gr * ld + c * 8 : (const bf16_t *)&zero16;
      __builtin_amdgcn_global_load_lds((gbl_void_t *)p, (lds_void_t *)(S + q * 512), 16, 0, 0);
    }
  }

  // Same tile, but row p (a token position of one request) is fetched from a paged cache
  // [blocks, Hkv, B, HD]: block id from the request's block table, B = 1 << bshift.  Positions at or
  // beyond row_end, and block ids outside [0, num_blocks), read zeros.
  static __device__ __forceinline__ void issue_paged(const bf16_t *cache, const int32_t *bt, int bshift, int Hkv, int kvh,
                                                     long long num_blocks, int row0, int row_end, bf16_t *S) {
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int q = wave + (NTHR / 64) * i;
      const int chunk = q * 64 + lane;
      const int lr = chunk / CPR, c = (chunk % CPR) ^ swz(lr);
      const int pos = row0 + lr;
      const bf16_t *p = (const bf16_t *)&zero16;
      if (pos < row_end) {
        const long long blk = bt[pos >> bshift];
        if (blk >= 0 && blk < num_blocks)
          p = cache + ((((size_t)blk * Hkv + kvh) << bshift) + (pos & ((1 << bshift) - 1))) * HD + c * 8;
      }
      __builtin_amdgcn_global_load_lds((gbl_void_t *)p, (lds_void_t *)(S + q * 512), 16, 0, 0);
    }
  }

  struct FragK { int base, sw; };
  static __device__ __forceinline__ FragK frag_k_init(int row) { return FragK{row * HD, swz(row)}; }
  // head-dim elements kk*16 + 8*half .. +7 of the row
  static __device__ __forceinline__ bf16x8_t frag_k(const bf16_t *S, const FragK &f, int kk, int half) {
    return *(const bf16x8_t *)(S + f.base + (((2 * kk + half) ^ f.sw) << 3));
  }

  struct FragT { int a0, a1; };
  // operand row = head-dim index r0 + lane%32 (r0 multiple of 32)
  static __device__ __forceinline__ FragT frag_t_init(int r0, int lane) {
    const int grp = lane >> 4, j = lane & 15;
    const int row = 8 * (grp >> 1) + (j >> 2);                       // + 16*kk (+4 for the second read)
    const int c = (r0 >> 3) + 2 * (grp & 1) + ((j & 3) >> 1);
    FragT f;
    f.a0 = row * HD + ((c ^ swz(row)) << 3) + 4 * (j & 1);
    f.a1 = (row + 4) * HD + ((c ^ swz(row + 4)) << 3) + 4 * (j & 1);
    return f;
  }
  static __device__ __forceinline__ bf16x8_t frag_t(const bf16_t *S, const FragT &f, int kk) {
    const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)(S + f.a0 + kk * 16 * HD));
    const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)(S + f.a1 + kk * 16 * HD));
    const s16x8_t v = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8_t, v);
  }
};

}  // namespace attn
