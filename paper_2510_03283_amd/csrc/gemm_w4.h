// 256x256x64 block tile on FOUR waves (2 x 2, wave tile 128x128), included by gemm.hip inside its
// anonymous namespace (it uses DirectStage's tile layouts and swizzles).
//
// One wave per SIMD owns all 512 registers of a lane: 256 accumulator registers (AGPRs) and 256
// VGPRs, of which 128 are two register sets that stage operand tiles on their way global -> VGPR
// -> LDS.  Compared with the 8-wave kernel (wave tile 128x64) a k step needs 0.5 instead of 0.75
// fragment reads per MFMA, the tiles reach LDS through 16-byte ds_writes (a quarter of the LDS time of
// a direct global->LDS load) and every global load has two tile times to land.  Nothing covers a
// stall of the only wave of a SIMD, so the loop is written as an explicit schedule: one fragment
// read or one "move" (wait for a staged register, ds_write it, request the same register again for
// the tile three ahead) behind single MFMAs, one barrier per k tile, and the first fragments of the
// next tile read behind that barrier under the last MFMAs of the current one.
//
// Operand loads are buffer loads whose resource spans the operand from its first to its last
// element: a load beyond the end returns zeros, which is the whole edge handling (rows past M or N
// of a k-contiguous operand, k past K of a row-contiguous one).  The loads are issued as asm and
// counted by the kernel (s_waitcnt vmcnt(31) before the ds_write of a register: the load that
// filled it two tile times ago is followed by 31 younger ones); left to the compiler, its wait
// insertion settles on half that distance for one of the two phases of the loop.  A staged
// register is touched by nothing but its load and its ds_write; the build checks the generated
// code for that.

template <int B, int E, class F>
__device__ __forceinline__ void static_for(F &&f) {
  if constexpr (B < E) {
    f(std::integral_constant<int, B>{});
    static_for<B + 1, E>(f);
  }
}

typedef __attribute__((address_space(3))) u32x4_t lds_u32x4_t;
typedef __attribute__((address_space(3))) char lds_char_t;

#define W4_SB __builtin_amdgcn_sched_barrier(0)
#define W4_IC(n) std::integral_constant<int, (n)>{}
#define W4_INL __attribute__((always_inline))

// Tile tt of a block's reduction -> where its operands come from: the low and high words of the operand
// bases (a buffer resource is {base lo, base hi, bytes, format}; u: the up weights in SwiGLU mode, else the
// B base again), the extent of B and the byte offsets of the tile's origin.  Bases differ by pass (hi / lo
// term) and by k segment.  Plain scalars, and a free function with every input passed by value: a resource
// that is the phi of two branches lands in vector registers, and written as a lambda the selections between
// captured variables become selections between their addresses and keep all of them in private memory.
struct W4Cur { uint32_t a0, a1, b0, b1, u0, u1, b_bytes, oa, ob; };
template <int LA, int LB>
__device__ __forceinline__ W4Cur w4_tile_src(int tt, int nk, int kt0, int m0, int n0, int N, int K, long long lda, long long ldb,
                                             const void *a_hi, const void *a_lo, const void *b_hi, const void *b_lo, const void *u_hi, const void *u_lo,
                                             int swiglu, int n_kseg, int ks_s1, int ks_s2, const void *ks_b0, const void *ks_b1, const void *ks_b2) {
  constexpr int BKT = 64;
  const int pass = tt >= 2 * nk ? 2 : (tt >= nk ? 1 : 0);
  const int k0 = (kt0 + tt - pass * nk) * BKT;
  W4Cur r;
  const uint64_t ab = (uint64_t)(pass == 1 ? a_lo : a_hi);
  r.a0 = (uint32_t)ab;
  r.a1 = (uint32_t)(ab >> 32) & 0xffffu;
  r.oa = (uint32_t)((LA == 0 ? (long long)m0 * lda + k0 : (long long)k0 * lda + m0) * 2);
  // the k range may be a concatenation whose segment ks takes its B rows from its own matrix
  const int ks = n_kseg > 1 ? (k0 >= ks_s1 ? 1 : 0) + (n_kseg > 2 && k0 >= ks_s2 ? 1 : 0) : 0;
  const int s0 = ks == 0 ? 0 : (ks == 1 ? ks_s1 : ks_s2), s1 = ks + 1 >= n_kseg ? K : (ks == 0 ? ks_s1 : ks_s2);
  const int kl = k0 - s0;
  const uint64_t bb = (uint64_t)(n_kseg > 1 ? (ks == 0 ? ks_b0 : (ks == 1 ? ks_b1 : ks_b2)) : (pass == 2 ? b_lo : b_hi));
  const uint64_t ub = swiglu ? (uint64_t)(pass == 2 ? u_lo : u_hi) : bb;
  r.b0 = (uint32_t)bb;
  r.b1 = (uint32_t)(bb >> 32) & 0xffffu;
  r.u0 = (uint32_t)ub;
  r.u1 = (uint32_t)(ub >> 32) & 0xffffu;
  r.b_bytes = (uint32_t)(2 * (LB == 0 ? (long long)(N - 1) * ldb + (s1 - s0) : (long long)(s1 - s0 - 1) * ldb + N));
  r.ob = (uint32_t)((LB == 0 ? (long long)n0 * ldb + kl : (long long)kl * ldb + n0) * 2);
  return r;
}
// The resources of a tile in scalar registers.
struct W4Src { u32x4_t qa, qb, qu; uint32_t oa, ob; };
__device__ __forceinline__ uint32_t w4_sgpr(uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)x); }
// dead: a request that only keeps the count of loads in flight constant (past the last tile) gets empty
// resources: its loads return zeros without going to memory.
__device__ __forceinline__ W4Src w4_resources(const W4Cur c, uint32_t a_bytes, bool dead = false) {
  W4Src r;
  a_bytes = dead ? 0u : a_bytes;
  const uint32_t b_bytes = dead ? 0u : c.b_bytes;
  r.qa = u32x4_t{w4_sgpr(c.a0), w4_sgpr(c.a1), w4_sgpr(a_bytes), 0x00020000u};
  r.qb = u32x4_t{w4_sgpr(c.b0), w4_sgpr(c.b1), w4_sgpr(b_bytes), 0x00020000u};
  r.qu = u32x4_t{w4_sgpr(c.u0), w4_sgpr(c.u1), w4_sgpr(b_bytes), 0x00020000u};
  r.oa = c.oa;
  r.ob = c.ob;
  return r;
}

// An accumulator element for the epilogue, read where it lives.  The accumulators stay in AGPRs from the loop to
// the end of the kernel; handed over as plain values, the register allocator copies whole 16-register blocks into
// VGPRs at the end of the loop for all epilogue variants at once, spills what does not fit and reloads a block
// per element between the stores (every reload a wait that drains the stores in flight).
__device__ __forceinline__ float w4_acc_rd(float a) {
  float v;
  asm("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
  return v;
}

template <int LA, int LB>
__global__ __launch_bounds__(256) void gemm_bf16_w4_kernel(const GemmParams p) {
  constexpr int BM = 256, BN = 256, BKT = 64, NTHR = 256, WGN = 2, WTM = 128, WTN = 128, TM = 4, TN = 4;
  using SA = DirectStage<BM, LA, BKT, 512>;    // tile layout, swizzle and fragment addressing
  using SB = DirectStage<BN, LB, BKT, 512>;
  constexpr int NL = BM * BKT / 8 / NTHR;      // 16-byte loads per lane and operand tile (8)
  constexpr int OPB = BM * BKT * 2;            // bytes of one operand tile (32 KB)
  // LDS: A stage 0 | A stage 1 | B stage 0 | B stage 1
  extern __shared__ __align__(16) unsigned char smem_raw[];
  lds_char_t *const lbase = (lds_char_t *)(lds_void_t *)smem_raw;

  // block -> tile: the mapping of gemm_bf16_dl_kernel
  const int n_ns_eff = p.swiglu ? 1 : p.n_ns;
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
      const int fy = (y - first_blk) & 7;
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
  const int swiglu = p.swiglu;
  const int m0 = mt_l * BM, n0 = swiglu ? nt_g * (BN / 2) : (nt_g - p.nt_start[s]) * BN;
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

  const int nk_all = (K + BKT - 1) / BKT;
  const int nk_per = (nk_all + (int)gridDim.y - 1) / (int)gridDim.y;
  const int kt0 = (int)blockIdx.y * nk_per;
  const int nk = max(0, min(nk_per, nk_all - kt0));
  const int n_it = nk * G.npass;
  const long long lda = p.lda, ldb = p.ldb;
  const int n_kseg = p.n_kseg;
  const int ks_s1 = p.kseg_start[1], ks_s2 = p.kseg_start[2];
  const void *const ks_b0 = p.kseg_b[0], *const ks_b1 = p.kseg_b[1], *const ks_b2 = p.kseg_b[2];

  const uint32_t a_bytes = (uint32_t)(2 * (LA == 0 ? (long long)(M - 1) * lda + K : (long long)(K - 1) * lda + M));
  const void *const a_hi = G.a[0], *const a_lo = G.npass >= 2 ? G.a[1] : G.a[0];
  const void *const b_hi = swiglu ? p.ns[0].b[0] : S.b[0], *const b_lo = G.npass >= 3 ? (swiglu ? p.ns[0].b[1] : S.b[1]) : b_hi;
  const void *const u_hi = swiglu ? p.ns[1].b[0] : b_hi, *const u_lo = swiglu && G.npass >= 3 ? p.ns[1].b[1] : u_hi;
  using Src = W4Src;
  auto tile_cur = [&](int tt) W4_INL -> W4Cur {
    return w4_tile_src<LA, LB>(tt, nk, kt0, m0, n0, N, K, lda, ldb, a_hi, a_lo, b_hi, b_lo, u_hi, u_lo, swiglu, n_kseg, ks_s1, ks_s2, ks_b0, ks_b1, ks_b2);
  };
  auto tile_src = [&](int tt) W4_INL -> Src { return w4_resources(tile_cur(tt), a_bytes); };
  // a tile that continues the k run of the one before it lies stepA / stepB bytes further on
  const uint32_t stepA = (uint32_t)(LA == 0 ? BKT * 2 : BKT * lda * 2), stepB = (uint32_t)(LB == 0 ? BKT * 2 : BKT * ldb * 2);

  // Byte offset of this lane's first load inside an operand tile; load x of a tile fetches the chunk
  // 256 x further on, which is strA (strB) bytes away in memory and keeps the swizzle phase.
  static_assert(256 % SA::CPR == 0 && 256 % SB::CPR == 0 && (256 / SA::CPR) % 4 == 0 && (256 / SB::CPR) % 4 == 0,
                "a step of 256 chunks must keep the swizzle phase");
  uint32_t offA, offB;
  {
    const int chunk = wave * 64 + lane;
    {
      const int lr = chunk / SA::CPR, pos = chunk % SA::CPR;
      if constexpr (LA == 0) {
        offA = (uint32_t)(((long long)lr * lda + (pos ^ ((lr / SA::RPB) % SA::CPR)) * 8) * 2);
      } else {
        const int c = SA::POW2 ? pos ^ ((lr & 3) << 2) : (pos + SA::CPR - 4 * (lr & 3)) % SA::CPR;
        offA = (uint32_t)(((long long)lr * lda + 8 * c) * 2);
      }
    }
    {
      const int lr = chunk / SB::CPR, pos = chunk % SB::CPR;
      if constexpr (LB == 0) {
        offB = (uint32_t)(((long long)lr * ldb + (pos ^ ((lr / SB::RPB) % SB::CPR)) * 8) * 2);
      } else {
        const int c = SB::POW2 ? pos ^ ((lr & 3) << 2) : (pos + SB::CPR - 4 * (lr & 3)) % SB::CPR;
        offB = (uint32_t)(((long long)lr * ldb + 8 * c) * 2);
      }
    }
  }
  const uint32_t strA = (uint32_t)(256 / SA::CPR * lda * 2), strB = (uint32_t)(256 / SB::CPR * ldb * 2);
  // k-contiguous B: loads 2u and 2u+1 are 32 rows apart, except in SwiGLU mode, where they fetch the gate and
  // the up rows of the same 32 hidden units out of two matrices
  const uint32_t strB_pair = swiglu ? strB : 2 * strB, strB_odd = swiglu ? 0u : strB;
  typename SA::FragAddr fa = SA::template frag_addr<TM>(wm * WTM, lane);
  typename SB::FragAddr fb = SB::template frag_addr<TN>(wn * WTN, lane);
  // The B stages start 64 KB into LDS, beyond the 16-bit offset field of an LDS instruction.  Their lane
  // addresses carry the 64 KB and are made opaque, so that stage and fragment offsets stay immediates (seen
  // as "lane part + constant" the compiler folds all constants into one and keeps a register per sum).
#pragma unroll
  for (int x = 0; x < 4; ++x) {
    fb.v[x] += 2 * OPB;
    asm volatile("" : "+v"(fb.v[x]));
  }
  const uint32_t wofs = (uint32_t)(wave * 1024 + lane * 16);     // load x of a tile sits at wofs + x * 4096
  uint32_t wofs_b = wofs + 2 * OPB;
  asm volatile("" : "+v"(wofs_b));

  u32x4_t ra[2][NL], rb[2][NL];        // register sets: tile t waits in set (t + 1) & 1
  u32x4_t fra[2][TM], frb[2][TN];      // fragments, double-buffered over k steps

  auto bload = [&](u32x4_t &dst, const u32x4_t &rs, uint32_t voff, uint32_t soff) W4_INL {
    asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen" : "=v"(dst) : "v"(voff), "s"(rs), "s"(soff));
  };
  // load x (0..7: A, 8..15: B) of the tile described by `src`.  SwiGLU mode: the B tile interleaves 32 gate
  // rows and the 32 up rows of the same hidden units; a load covers 8 rows of one of the two.
  auto request = [&](auto SET, auto X, const Src &src) W4_INL {
    constexpr int set = decltype(SET)::value, x = decltype(X)::value;
    if constexpr (x < NL) {
      bload(ra[set][x], src.qa, offA, src.oa + x * strA);
    } else {
      constexpr int y = x - NL;
      if constexpr (LB == 0) bload(rb[set][y], (y & 1) ? src.qu : src.qb, offB, src.ob + (y >> 1) * strB_pair + (y & 1) * strB_odd);
      else bload(rb[set][y], src.qb, offB, src.ob + y * strB);
    }
  };
  auto stage_write = [&](auto SET, auto X, auto ST) W4_INL {
    constexpr int set = decltype(SET)::value, x = decltype(X)::value, st = decltype(ST)::value;
    if constexpr (x < NL) *(lds_u32x4_t *)(lbase + wofs + st * OPB + x * 4096) = ra[set][x];
    else *(lds_u32x4_t *)(lbase + wofs_b + st * OPB + (x - NL) * 4096) = rb[set][x - NL];
  };
  // fragment f (0..3: A rows, 4..7: B columns) of k step kk out of stage st into fragment buffer nb
  auto read1 = [&](auto ST, auto KK, auto NB, auto FF) W4_INL {
    constexpr int st = decltype(ST)::value, kk = decltype(KK)::value, nb = decltype(NB)::value, f = decltype(FF)::value;
    if constexpr (f < TM) {
      if constexpr (LA == 0) {
        fra[nb][f] = *(lds_u32x4_t *)(lbase + fa.v[kk] + st * OPB + f * 32 * BKT * 2);
      } else {
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)(lbase + fa.v[f] + st * OPB + kk * 16 * BM * 2));
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)(lbase + fa.v[f] + st * OPB + kk * 16 * BM * 2 + 4 * BM * 2));
        const u32x2_t l2 = __builtin_bit_cast(u32x2_t, lo), h2 = __builtin_bit_cast(u32x2_t, hi);
        fra[nb][f] = u32x4_t{l2[0], l2[1], h2[0], h2[1]};
      }
    } else {
      constexpr int j = f - TM;
      if constexpr (LB == 0) {
        frb[nb][j] = *(lds_u32x4_t *)(lbase + fb.v[kk] + st * OPB + j * 32 * BKT * 2);
      } else {
        const s16x4_t lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)(lbase + fb.v[j] + st * OPB + kk * 16 * BN * 2));
        const s16x4_t hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4_t *)(lbase + fb.v[j] + st * OPB + kk * 16 * BN * 2 + 4 * BN * 2));
        const u32x2_t l2 = __builtin_bit_cast(u32x2_t, lo), h2 = __builtin_bit_cast(u32x2_t, hi);
        frb[nb][j] = u32x4_t{l2[0], l2[1], h2[0], h2[1]};
      }
    }
  };
  auto mfma1 = [&](auto KK, auto Q) W4_INL {
    constexpr int kk = decltype(KK)::value, q = decltype(Q)::value, i = q / TN, j = q % TN;
    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, fra[kk & 1][i]), __builtin_bit_cast(bf16x8_t, frb[kk & 1][j]), acc[i][j], 0, 0, 0);
  };

  if (n_it <= 0) {
    // an empty k slice of a split reduction (fp32 partial sums, no residual): its tile is zeros.  Kept apart
    // from the main path so that the accumulators are not a phi around the loop.
    float *const zp = (float *)G.c + (long long)blockIdx.y * p.c_split_stride + S.c_col;
    for (int e = threadIdx.x; e < BM * BN; e += NTHR) {
      const int row = m0 + e / BN, col = n0 + e % BN;
      if (row < M && col < N) zp[(long long)row * p.ldc + col] = 0.f;
    }
    return;
  }
  const int n_run = max(n_it, 3);      // tile times: at least one turn of the loop and one tile behind it
  int rq_tt;      // the tile requested last, and where it comes from
  W4Cur rq;
  {
    // prologue: tile 0 -> set 1 -> stage 0; tile 1 -> set 0; tile 2 -> set 1.  Tiles past the last repeat
    // the last one (their data is never multiplied): the loop's wait counts assume every request is issued.
    {
      const Src s0 = tile_src(0);
      static_for<0, 2 * NL>([&](auto X) W4_INL { request(W4_IC(1), X, s0); });
      W4_SB;
      const Src s1 = w4_resources(tile_cur(min(1, n_it - 1)), a_bytes, n_it < 2);
      static_for<0, 2 * NL>([&](auto X) W4_INL { request(W4_IC(0), X, s1); });
      W4_SB;
      wait_vmcnt<2 * NL>();      // tile 0 is in
      W4_SB;
      static_for<0, 2 * NL>([&](auto X) W4_INL { stage_write(W4_IC(1), X, W4_IC(0)); });
      W4_SB;
      rq_tt = min(2, n_it - 1);
      rq = tile_cur(rq_tt);
      const Src s2 = w4_resources(rq, a_bytes, n_it < 3);
      static_for<0, 2 * NL>([&](auto X) W4_INL { request(W4_IC(1), X, s2); });
      W4_SB;
      __syncthreads();
      static_for<0, TM + TN>([&](auto F) W4_INL { read1(W4_IC(0), W4_IC(0), W4_IC(0), F); });
      W4_SB;
    }
    // Tile time t (phase ph = t & 1): multiply tile t out of stage ph; move tile t+1 from register set ph
    // into stage ph^1 (free since the barrier of tile time t-1), re-requesting each register right after
    // its ds_write for tile t+3; barrier behind the first MFMA of the last k step; the first fragments of
    // tile t+1 behind the barrier.
    auto phase = [&](auto PH, auto TAIL, int t) W4_INL {
      constexpr int ph = decltype(PH)::value;
      constexpr bool tail = decltype(TAIL)::value;
      // the next request: tile t + 3, or the last tile again.  Only a change of pass or of k segment takes
      // the full computation.
      bool dead = false;
      if (!tail && rq_tt >= n_it - 1) dead = true;
      if (!tail && rq_tt < n_it - 1) {
        ++rq_tt;
        const int kq = (kt0 + rq_tt) * BKT;      // (k segments exclude passes)
        if (rq_tt == nk || rq_tt == 2 * nk || (n_kseg > 1 && (kq == ks_s1 || kq == ks_s2))) {
          rq = tile_cur(rq_tt);
        } else {
          rq.oa += stepA;
          rq.ob += stepB;
        }
      }
      const Src src = w4_resources(rq, a_bytes, dead);
      // (the tiles behind the loop request nothing: what they would request lies past the last tile, and a
      // load still in flight when control leaves this code could land in a register that holds something else
      // by then; the last of them moves nothing either)
      auto move = [&](auto X) W4_INL {
        if constexpr (!tail) {
          wait_vmcnt<4 * NL - 1>();      // the load that filled this register is followed by 31 younger ones
          W4_SB;
        }
        if constexpr (!(tail && ph == 1)) stage_write(W4_IC(ph), X, W4_IC(ph ^ 1));
        if constexpr (!tail) {
          W4_SB;
          request(W4_IC(ph), X, src);
        }
      };
      // k steps 0..2: behind fourteen of the sixteen MFMAs either one fragment read of the next step or one move,
      // the two kinds interleaved (r m r r m r - r m r m r m r m -; 16 moves over the three steps).  Measured
      // against other orders on one box: all eight reads first and the six moves behind them is 1 - 4 % slower on
      // every shape, moves first 1 - 4 % slower still.  (One heavy instruction behind every MFMA - all ds_writes
      // first, the requests behind them, the last eight in k step 3 - is 1 - 2 % faster than reads-then-moves on
      // long reductions and makes the first k tiles of every output tile slower.)
      static_for<0, 3>([&](auto KK) W4_INL {
        constexpr int kk = decltype(KK)::value;
        static_for<0, 16>([&](auto Q) W4_INL {
          constexpr int q = decltype(Q)::value;
          mfma1(KK, Q);
          // what follows MFMA q of a k step: fragment RD[q] of the next step, or move MV[q] of this step's six
          constexpr int RD[16] = {0, -1, 1, 2, -1, 3, -1, 4, -1, 5, -1, 6, -1, 7, -1, -1};
          constexpr int MV[16] = {-1, 0, -1, -1, 1, -1, -1, -1, 2, -1, 3, -1, 4, -1, 5, -1};
          if constexpr (RD[q] >= 0) { read1(W4_IC(ph), W4_IC(kk + 1), W4_IC((kk + 1) & 1), W4_IC(RD[q])); W4_SB; }
          if constexpr (MV[q] >= 0 && kk * 6 + MV[q] < 2 * NL) { W4_SB; move(W4_IC(kk * 6 + MV[q])); W4_SB; }
        });
      });
      mfma1(W4_IC(3), W4_IC(0)); W4_SB;
      __syncthreads();
      W4_SB;
      static_for<1, 16>([&](auto Q) W4_INL {
        constexpr int q = decltype(Q)::value;
        if constexpr (q <= 8) read1(W4_IC(ph ^ 1), W4_IC(0), W4_IC(0), W4_IC(q - 1));
        mfma1(W4_IC(3), Q); W4_SB;
      });
      // The compiler does not know which registers have a load in flight, and where control leaves the loop it
      // may copy or spill what is live there.  So the loop's last iteration ends with a wait for all loads (the
      // pipeline runs empty once per output tile), and the code behind the loop issues none.
      if constexpr (!tail && ph == 1) {
        if (t + 3 >= n_run) {
          wait_vmcnt<0>();
          W4_SB;
        }
      }
    };
    // The loop proper has no exit but its back edge; the last one or two tiles run behind it.  It always runs at
    // least once: a reduction of one or two tiles is padded with empty tiles (zeros, requested from empty
    // resources).  With a way around the loop the accumulators reach the code behind it in two register
    // assignments, and the loop's exit pays for the difference with a permutation of all of them.
    int t = 0;
    do {
      phase(W4_IC(0), std::false_type{}, t);
      phase(W4_IC(1), std::false_type{}, t + 1);
      t += 2;
    } while (t + 2 < n_run);
    phase(W4_IC(0), std::true_type{}, t);
    if (t + 1 < n_run) phase(W4_IC(1), std::true_type{}, t + 1);
  }

  // Epilogue.  Accumulator register r of block (i, j) holds row 8 (r / 4) + 4 (lane / 32) + r % 4 and column
  // lane % 32 of the 32x32 block.  Every access is a buffer instruction on a view of the wave's part of the
  // matrix (from its first row and column on, as many bytes as its existing rows take): the address is
  // "view + uniform row offset + lane offset".  The row offset is one scalar that walks down the rows (from one
  // register to the next the row index grows by 1, 1, 1, 5; by 2, 6 where registers are handled in pairs), the
  // lane offset one register per column block, and that is all the address arithmetic there is.  Edges need no
  // code: an access to a row past the last is out of the view's range, which the hardware drops (a load
  // returns zero), a lane whose column does not exist carries an offset beyond any view, and an output that was
  // not asked for is an empty view.
  // (no lambda below may name p, G or S: captured by reference the kernel arguments are copied to private memory)
  // (the reads of the accumulators are asm, which the compiler's hazard handling does not look into: the wait
  // states between the last MFMA and the first read of its result are given here)
  asm volatile("s_nop 15\n\ts_nop 15");
  W4_SB;
  const int rk = p.resid_kind, obf = p.out_bf16;
  void *const Cp = G.c;
  const void *const Rp = G.resid;
  const int c_col = S.c_col;
  const long long ldc = p.ldc, ldr = p.ldr;
  const bool odd = lane & 1;
  const int row_u = m0 + wm * WTM;                                  // the wave's first row
  const int rows_v = max(0, min(WTM, M - row_u));                   // how many of its rows exist
  const int lrow = 4 * (lane >> 5), lcol = lane & 31;
  constexpr uint32_t OUT = 0x80000000u;                             // lane offset of a column that does not exist
  auto view = [](const void *base, long long bytes) W4_INL {
    return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, (int)bytes, 0x00020000);
  };
  // (stores carry the non-temporal hint: the outputs are not read again by this launch, and kept out of the way of
  // the operand panels in L2 the two-pass shapes run 1.7 % faster; one-pass shapes do not change)
  auto store32 = [](uint32_t w, __amdgpu_buffer_rsrc_t q, uint32_t voff, uint32_t soff) W4_INL {
    __builtin_amdgcn_raw_buffer_store_b32(w, q, (int)voff, (int)soff, 2);
  };
  auto swap_pair = [&](float mine_r, float mine_r1) W4_INL -> float {     // the partner's value for the row this lane stores
    const float send = odd ? mine_r : mine_r1;
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(send), 0xB1, 0xF, 0xF, true));
  };
  if (swiglu) {
    if constexpr (LA == 0 && LB == 0) {
      // column blocks (0, 1) and (2, 3) of a wave are G and U of the same 32 hidden units
      const int F = N;
      bf16_t *const hi = (bf16_t *)Cp, *const lo = (bf16_t *)G.c_lo, *const gu = (bf16_t *)G.c_gu;
      const int f_u = n0 + wn * (WTN / 2);
      // Stores of full 128-byte lines.  After the pair swap a lane holds the packed pair (fc, fc + 1) of row
      // (row + odd) for each of the wave's two unit blocks (jj = 0, 1), in the row half lane / 32 selects.  One
      // v_permlane32_swap of the two blocks' words gives {lower lanes: block 0, upper lanes: block 1} of
      // row half 0 in one register and the same of row half 1 in the other: a store then covers 64 units
      // (128 bytes) of two rows instead of 32 units of four.
      const int col_l = lane - (odd ? 1 : 0);                      // lane part of the unit index (blocks are 32 apart)
      const int row_l = odd ? 1 : 0;                               // lane part of the row
      const bool okc = f_u + col_l < F;
      // lane offsets for row half 0 and (four rows on) row half 1; U lies F units behind G
      uint32_t vh[2], vg[2], vu[2];
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        vh[hh] = okc ? (uint32_t)((int)((row_l + 4 * hh) * ldc) + col_l) * 2u : OUT;
        vg[hh] = okc ? (uint32_t)((row_l + 4 * hh) * 2 * F + col_l) * 2u : OUT;
        vu[hh] = okc ? vg[hh] + (uint32_t)F * 2u : OUT;
      }
      const auto qh = view(hi + (long long)row_u * ldc + f_u, rows_v * ldc * 2);
      const auto ql = view(lo + (long long)row_u * ldc + f_u, lo ? rows_v * ldc * 2 : 0);
      const auto qg = view(gu + (long long)row_u * 2 * F + f_u, gu ? (long long)rows_v * F * 4 : 0);
      // (row strides go through w4_sgpr: a stride that shares a subexpression with a lane offset is otherwise
      // computed in vector registers, and a vector register as the scalar offset of a buffer instruction
      // becomes a loop over its distinct values)
      const uint32_t h2r = w4_sgpr((uint32_t)(ldc * 4)), h6r = w4_sgpr((uint32_t)(ldc * 12)), g2r = w4_sgpr((uint32_t)F * 8u), g6r = w4_sgpr((uint32_t)F * 24u);      // 2 and 6 rows
      // KIND 0: only hm (inference rows); 1: hm in two terms and G, U kept (fine-tune rows)
      auto emit = [&](auto KIND) W4_INL {
        constexpr int kind = decltype(KIND)::value;
        uint32_t sh = 0, sg = 0;      // row offsets in hm (both terms) and in G|U
        static_for<0, TM>([&](auto I) W4_INL {
          constexpr int i = decltype(I)::value;
          static_for<0, 8>([&](auto R2) W4_INL {
            constexpr int r = 2 * decltype(R2)::value;
            uint32_t wh[2], wl[2], wg[2], wu[2];
            static_for<0, 2>([&](auto JJ) W4_INL {
              constexpr int jj = decltype(JJ)::value;
              const float g2[2] = {w4_acc_rd(acc[i][2 * jj][r]), w4_acc_rd(acc[i][2 * jj][r + 1])};
              const float u2[2] = {w4_acc_rd(acc[i][2 * jj + 1][r]), w4_acc_rd(acc[i][2 * jj + 1][r + 1])};
              float h2[2];
#pragma unroll
              for (int e = 0; e < 2; ++e) h2[e] = g2[e] * __builtin_amdgcn_rcpf(1.0f + __expf(-g2[e])) * u2[e];
              const float hp = swap_pair(h2[0], h2[1]);
              split_pk_bf16(odd ? hp : h2[0], odd ? h2[1] : hp, wh[jj], wl[jj]);
              if constexpr (kind != 0) {
                const float gp = swap_pair(g2[0], g2[1]), up = swap_pair(u2[0], u2[1]);
                wg[jj] = cvt_pk_bf16(odd ? gp : g2[0], odd ? g2[1] : gp);
                wu[jj] = cvt_pk_bf16(odd ? up : u2[0], odd ? u2[1] : up);
              }
            });
            // row halves: words [0] belong to rows (row + row_l), words [1] to the rows four further on
            const u32x2_t s_h = __builtin_amdgcn_permlane32_swap(wh[0], wh[1], false, false);
            static_for<0, 2>([&](auto H) W4_INL { store32(s_h[decltype(H)::value], qh, vh[decltype(H)::value], sh); });
            if constexpr (kind != 0) {
              const u32x2_t s_l = __builtin_amdgcn_permlane32_swap(wl[0], wl[1], false, false);
              const u32x2_t s_g = __builtin_amdgcn_permlane32_swap(wg[0], wg[1], false, false);
              const u32x2_t s_u = __builtin_amdgcn_permlane32_swap(wu[0], wu[1], false, false);
              static_for<0, 2>([&](auto H) W4_INL {
                constexpr int hh = decltype(H)::value;
                store32(s_l[hh], ql, vh[hh], sh);
                store32(s_g[hh], qg, vg[hh], sg);
                store32(s_u[hh], qg, vu[hh], sg);
              });
            }
            sh += (r & 2) ? h6r : h2r;
            sg += (r & 2) ? g6r : g2r;
          });
          W4_SB;
        });
      };
      if (!lo && !gu) emit(W4_IC(0));
      else emit(W4_IC(1));
    }
    return;
  }
  const int col_u = n0 + wn * WTN;                                  // the wave's first column
  if (G.rope) {
    if constexpr (LA == 0 && LB == 0) {
      // Rotary embedding and operand split in the epilogue of the QKV product: the wave's 128 columns are one head
      // (head dimension 128), so element i of the head sits in column blocks 0, 1 and its partner i + 64 in the
      // same register of blocks 2, 3.  (cos, sin) of (row, i) come from the group's table; the rotated (Q, K) or
      // plain (V) values leave as two bf16 terms through the pair and half swaps of the packed bf16 stores.
      const int rot = S.rope_rot;
      bf16_t *const ohi = (bf16_t *)S.rope_hi, *const olo = (bf16_t *)S.rope_lo;
      const int col_l = lane - (odd ? 1 : 0), row_l = odd ? 1 : 0;
      uint32_t vo[2][2];      // lane offsets of the stores by row half and block pair (output rows are N wide)
#pragma unroll
      for (int hh = 0; hh < 2; ++hh)
#pragma unroll
        for (int jp = 0; jp < 2; ++jp)
          vo[hh][jp] = col_u + jp * 64 + col_l < N ? (uint32_t)((row_l + 4 * hh) * N + col_l + jp * 64) * 2u : OUT;
      const uint32_t vt[2] = {(uint32_t)(lrow * 64 + lcol) * 8u, (uint32_t)(lrow * 64 + 32 + lcol) * 8u};      // table, blocks 0 and 1
      const auto qh = view(ohi + (long long)row_u * N + col_u, (long long)rows_v * N * 2);
      const auto ql = view(olo + (long long)row_u * N + col_u, olo ? (long long)rows_v * N * 2 : 0);
      const auto qt = view(p.rope_cs + (long long)row_u * 128, (long long)rows_v * 512);
      const uint32_t o2r = w4_sgpr((uint32_t)N * 4u), o6r = w4_sgpr((uint32_t)N * 12u);      // 2 and 6 output rows
      uint32_t so = 0, st = 0;      // row offsets of the outputs and of the table
      static_for<0, TM>([&](auto I) W4_INL {
        constexpr int i = decltype(I)::value;
        u32x2_t cs[16][2];      // the table entries of the block row's 16 registers, requested together
        {
          uint32_t q = st;
          static_for<0, 16>([&](auto R) W4_INL {
            constexpr int r = decltype(R)::value;
            static_for<0, 2>([&](auto J) W4_INL { cs[r][decltype(J)::value] = __builtin_amdgcn_raw_buffer_load_b64(qt, (int)vt[decltype(J)::value], (int)q, 0); });
            q += (r & 3) == 3 ? 2560u : 512u;
          });
          st += 32u * 512u;
        }
        W4_SB;
        static_for<0, 8>([&](auto R2) W4_INL {
          constexpr int r2 = decltype(R2)::value, r = 2 * r2;
          float v[TN][2];
          static_for<0, TN>([&](auto J) W4_INL {
            constexpr int j = decltype(J)::value;
            v[j][0] = w4_acc_rd(acc[i][j][r]);
            v[j][1] = w4_acc_rd(acc[i][j][r + 1]);
          });
          if (rot) {
#pragma unroll
            for (int j = 0; j < 2; ++j)
#pragma unroll
              for (int e = 0; e < 2; ++e) {
                const float c = __uint_as_float(cs[r + e][j][0]), sn = __uint_as_float(cs[r + e][j][1]);
                const float a = v[j][e], b = v[j + 2][e];
                v[j][e] = a * c - b * sn;
                v[j + 2][e] = b * c + a * sn;
              }
          }
          uint32_t wh[TN], wl[TN];
#pragma unroll
          for (int j = 0; j < TN; ++j) {
            const float vx = swap_pair(v[j][0], v[j][1]);
            split_pk_bf16(odd ? vx : v[j][0], odd ? v[j][1] : vx, wh[j], wl[j]);
          }
          static_for<0, 2>([&](auto JP) W4_INL {
            constexpr int jp = decltype(JP)::value;
            const u32x2_t s_h = __builtin_amdgcn_permlane32_swap(wh[2 * jp], wh[2 * jp + 1], false, false);
            const u32x2_t s_l = __builtin_amdgcn_permlane32_swap(wl[2 * jp], wl[2 * jp + 1], false, false);
            static_for<0, 2>([&](auto H) W4_INL {
              constexpr int hh = decltype(H)::value;
              store32(s_h[hh], qh, vo[hh][jp], so);
              store32(s_l[hh], ql, vo[hh][jp], so);
            });
          });
          so += (r2 & 1) ? o6r : o2r;
        });
        W4_SB;
      });
    }
    return;
  }
  const long long c_col0 = c_col + (long long)blockIdx.y * p.c_split_stride;
  if (p.swiglu_bwd) {
    if constexpr (LA == 0 && LB == 1) {
      // SwiGLU backward in the epilogue of dHm = dY Wd: the tile of dHm never leaves the registers.  With G and U of
      // the forward (bf16 [M, 2F], G | U) it becomes dG = dHm U s (1 + G (1 - s)) and dU = dHm G s, s = sigmoid(G),
      // written as bf16 [M, 2F] (dG | dU) - the same layout, so G, U, dG and dU of an element pair share one lane
      // offset (U and dU lie F columns further on).  The pair and half swaps of the packed bf16 stores are done on
      // the fp32 values, so that a lane computes on the two neighbouring columns it loads and stores as one word.
      const int F = N;
      const int col_l = lane - (odd ? 1 : 0), row_l = odd ? 1 : 0;
      uint32_t vg[2][TN / 2], vu[2][TN / 2];      // lane offsets by row half and block pair, G / dG and U / dU
#pragma unroll
      for (int hh = 0; hh < 2; ++hh)
#pragma unroll
        for (int jp = 0; jp < TN / 2; ++jp) {
          const bool ok = col_u + jp * 64 + col_l < F;
          vg[hh][jp] = ok ? (uint32_t)((row_l + 4 * hh) * 2 * F + col_l + jp * 64) * 2u : OUT;
          vu[hh][jp] = ok ? vg[hh][jp] + (uint32_t)F * 2u : OUT;
        }
      const auto qo = view((bf16_t *)Cp + (long long)row_u * 2 * F + col_u, (long long)rows_v * F * 4);
      const auto qi = view((const bf16_t *)G.c_gu + (long long)row_u * 2 * F + col_u, (long long)rows_v * F * 4);
      const uint32_t s2r = w4_sgpr((uint32_t)F * 8u), s6r = w4_sgpr((uint32_t)F * 24u);      // 2 and 6 rows
      uint32_t sc = 0;
      static_for<0, TM>([&](auto I) W4_INL {
        constexpr int i = decltype(I)::value;
        // G and U of the 32 rows of block row i are requested together (nothing else covers the latency)
        uint32_t gw[8][TN / 2][2], uw[8][TN / 2][2];
        {
          uint32_t q = sc;
          static_for<0, 8>([&](auto R2) W4_INL {
            constexpr int r2 = decltype(R2)::value;
            static_for<0, TN / 2>([&](auto JP) W4_INL {
              static_for<0, 2>([&](auto H) W4_INL {
                constexpr int jp = decltype(JP)::value, hh = decltype(H)::value;
                gw[r2][jp][hh] = __builtin_amdgcn_raw_buffer_load_b32(qi, (int)vg[hh][jp], (int)q, 0);
                uw[r2][jp][hh] = __builtin_amdgcn_raw_buffer_load_b32(qi, (int)vu[hh][jp], (int)q, 0);
              });
            });
            q += (r2 & 1) ? s6r : s2r;
          });
        }
        W4_SB;
        static_for<0, 8>([&](auto R2) W4_INL {
          constexpr int r2 = decltype(R2)::value, r = 2 * r2;
          static_for<0, TN / 2>([&](auto JP) W4_INL {
            constexpr int jp = decltype(JP)::value;
            float x0[2], x1[2];      // the lane's column pair of dHm, by block of the pair
            static_for<0, 2>([&](auto JB) W4_INL {
              constexpr int jb = decltype(JB)::value, j = 2 * jp + jb;
              const float va = w4_acc_rd(acc[i][j][r]), vb = w4_acc_rd(acc[i][j][r + 1]);
              const float vx = swap_pair(va, vb);
              x0[jb] = odd ? vx : va;
              x1[jb] = odd ? vb : vx;
            });
            const u32x2_t t0 = __builtin_amdgcn_permlane32_swap(__float_as_uint(x0[0]), __float_as_uint(x0[1]), false, false);
            const u32x2_t t1 = __builtin_amdgcn_permlane32_swap(__float_as_uint(x1[0]), __float_as_uint(x1[1]), false, false);
            static_for<0, 2>([&](auto H) W4_INL {
              constexpr int hh = decltype(H)::value;
              const float dh[2] = {__uint_as_float(t0[hh]), __uint_as_float(t1[hh])};
              const uint32_t g2 = gw[r2][jp][hh], u2 = uw[r2][jp][hh];
              float dg[2], du[2];
#pragma unroll
              for (int e = 0; e < 2; ++e) {
                const float g = e ? __uint_as_float(g2 & 0xffff0000u) : __uint_as_float(g2 << 16);
                const float u = e ? __uint_as_float(u2 & 0xffff0000u) : __uint_as_float(u2 << 16);
                const float sg = __builtin_amdgcn_rcpf(1.0f + __expf(-g));
                du[e] = dh[e] * g * sg;
                dg[e] = dh[e] * u * sg * (1.0f + g * (1.0f - sg));
              }
              store32(cvt_pk_bf16(dg[0], dg[1]), qo, vg[hh][jp], sc);
              store32(cvt_pk_bf16(du[0], du[1]), qo, vu[hh][jp], sc);
            });
          });
          sc += (r2 & 1) ? s6r : s2r;
        });
        W4_SB;
      });
    }
    return;
  }
  if (obf) {
    // packed bf16 (even column count and offset, no residual): neighbouring lanes (columns c, c+1) swap one
    // value of a register pair (rows r, r+1); the even lane then holds columns (c, c+1) of row r, the odd lane
    // columns (c-1, c) of row r+1.  The words of two neighbouring column blocks go through v_permlane32_swap
    // (see the SwiGLU stores): a store covers 64 columns (128 bytes) of two rows.
    const int col_l = lane - (odd ? 1 : 0), row_l = odd ? 1 : 0;
    uint32_t vp[2][TN / 2];      // lane offsets by row half and block pair
#pragma unroll
    for (int hh = 0; hh < 2; ++hh)
#pragma unroll
      for (int jp = 0; jp < TN / 2; ++jp)
        vp[hh][jp] = col_u + jp * 64 + col_l < N ? (uint32_t)((int)((row_l + 4 * hh) * ldc) + col_l + jp * 64) * 2u : OUT;
    const auto qc = view((bf16_t *)Cp + (long long)row_u * ldc + c_col + col_u, rows_v * ldc * 2);
    const uint32_t p2r = w4_sgpr((uint32_t)(ldc * 4)), p6r = w4_sgpr((uint32_t)(ldc * 12));      // 2 and 6 rows
    uint32_t sc = 0;
    static_for<0, TM>([&](auto I) W4_INL {
      static_for<0, 8>([&](auto R2) W4_INL {
        constexpr int i = decltype(I)::value, r = 2 * decltype(R2)::value;
        static_for<0, TN / 2>([&](auto JP) W4_INL {
          constexpr int jp = decltype(JP)::value;
          uint32_t w[2];
          static_for<0, 2>([&](auto JB) W4_INL {
            constexpr int jb = decltype(JB)::value, j = 2 * jp + jb;
            const float va = w4_acc_rd(acc[i][j][r]), vb = w4_acc_rd(acc[i][j][r + 1]);
            const float vx = swap_pair(va, vb);
            w[jb] = cvt_pk_bf16(odd ? vx : va, odd ? vb : vx);
          });
          const u32x2_t sw = __builtin_amdgcn_permlane32_swap(w[0], w[1], false, false);
          static_for<0, 2>([&](auto H) W4_INL { store32(sw[decltype(H)::value], qc, vp[decltype(H)::value][jp], sc); });
        });
        sc += (r & 2) ? p6r : p2r;
      });
      W4_SB;
    });
    return;
  }
  // fp32 output; RES 0: no residual, 1: + fp32 residual (projections onto an fp32 stream, weight gradients that
  // accumulate), 2: + bf16 residual.  The residuals of eight blocks are requested together before the first is
  // added: with one wave per SIMD nothing else covers the latency of a request.
  auto emit = [&](auto RES) W4_INL {
    constexpr int res = decltype(RES)::value, rsz = res == 2 ? 2 : 4;
    uint32_t vc[TN], vr[TN];      // lane offsets by column block, in C and in the residual
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const bool ok = col_u + j * 32 + lcol < N;
      vc[j] = ok ? (uint32_t)((int)(lrow * ldc) + lcol + j * 32) * 4u : OUT;
      vr[j] = ok ? (uint32_t)((int)(lrow * ldr) + lcol + j * 32) * (uint32_t)rsz : OUT;
    }
    const auto qc = view((char *)Cp + ((long long)row_u * ldc + c_col0 + col_u) * 4, rows_v * ldc * 4);
    const auto qr = view((const char *)Rp + ((long long)row_u * ldr + c_col0 + col_u) * rsz, res ? rows_v * ldr * rsz : 0);
    const uint32_t c1 = w4_sgpr((uint32_t)(ldc * 4)), c5 = w4_sgpr((uint32_t)(ldc * 20)), c64 = w4_sgpr((uint32_t)(ldc * 256));
    const uint32_t r1 = w4_sgpr((uint32_t)(ldr * rsz)), r5 = w4_sgpr((uint32_t)(ldr * (5 * rsz))), r64 = w4_sgpr((uint32_t)(ldr * (64 * rsz)));
    uint32_t sc = 0, sr = 0;      // row offsets of the current 64-row half
    static_for<0, TM / 2>([&](auto IH) W4_INL {
      constexpr int ih = decltype(IH)::value;
      float rv[2][16][TN];
      if constexpr (res != 0) {
        static_for<0, TN>([&](auto J) W4_INL {
          constexpr int j = decltype(J)::value;
          uint32_t q = sr;
          static_for<0, 32>([&](auto IR) W4_INL {
            constexpr int ii = decltype(IR)::value / 16, r = decltype(IR)::value % 16;
            if constexpr (res == 1) rv[ii][r][j] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(qr, (int)vr[j], (int)q, 0));
            else rv[ii][r][j] = bf2f(__builtin_amdgcn_raw_buffer_load_b16(qr, (int)vr[j], (int)q, 0));
            q += (r & 3) == 3 ? r5 : r1;
          });
        });
        sr += r64;
        W4_SB;
      }
      static_for<0, TN>([&](auto J) W4_INL {
        constexpr int j = decltype(J)::value;
        uint32_t q = sc;
        static_for<0, 32>([&](auto IR) W4_INL {
          constexpr int ii = decltype(IR)::value / 16, r = decltype(IR)::value % 16, i = 2 * ih + ii;
          float v = w4_acc_rd(acc[i][j][r]);
          if constexpr (res != 0) v += rv[ii][r][j];
          store32(__builtin_bit_cast(uint32_t, v), qc, vc[j], q);
          q += (r & 3) == 3 ? c5 : c1;
        });
        W4_SB;
      });
      sc += c64;
    });
  };
  if (rk == 0) emit(W4_IC(0));
  else if (rk == 1) emit(W4_IC(1));
  else emit(W4_IC(2));
}

// Operand views must fit the 32-bit byte offsets of a buffer load, and 128 rows of an output or residual the
// 31 bits of an offset inside a wave's view.  bf16 output is stored in column pairs and takes no residual here.
template <int LA, int LB>
bool w4_fits(const GemmParams &p) {
  const long long lim = (1ll << 32) - 65536;
  for (int g = 0; g < p.n_mg; ++g) {
    const long long rows = LA == 0 ? p.mg[g].M : p.K;
    if (rows * p.lda * 2 >= lim) return false;
  }
  for (int s = 0; s < p.n_ns; ++s) {
    const long long rows = LB == 0 ? p.ns[s].N : p.K;
    if (rows * p.ldb * 2 >= lim) return false;
    if (p.out_bf16 && !p.swiglu && ((p.ns[s].N & 1) || (p.ns[s].c_col & 1))) return false;
    if (p.swiglu && (p.ns[s].N & 1)) return false;
  }
  if (p.out_bf16 && !p.swiglu && p.resid_kind != 0) return false;
  if (p.swiglu_bwd && !(LA == 0 && LB == 1)) return false;
  for (int g = 0; g < p.n_mg; ++g)
    if (p.mg[g].rope && !(LA == 0 && LB == 0)) return false;
  if (p.ldc >= (1ll << 21) || p.ldr >= (1ll << 21)) return false;
  return true;
}
