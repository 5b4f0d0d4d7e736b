// C ABI of the hybrid-iteration library: argument validation, workspace layout, launch sequences.
#include <cmath>
#include <cstdio>
#include <cstdlib>
#include <algorithm>
#include <cstring>
#include <string>
#include <vector>

#include "../../include/mace.h"
#include "gemm.h"
#include "kernels.h"

// Optional in-stream timing: one event before every launch and one at the end of a call, so the
// time of launch i is event[i+1] - event[i] on the stream the kernels run on.
struct ProfMark {
  int tag;         // index into PROF_TAGS, or -1 for a closing event
  int chain;       // 0 = the caller's stream, 1 = the side stream
  double flops, bytes;
};
// The weight-gradient GEMMs of the backward pass depend on nothing that follows them, so they run
// on a side stream of the context (same priority, non-blocking) forked from and joined back into
// the caller's stream with events inside each call: they fill the CUs that the small dX GEMMs and
// the elementwise kernels of the main chain leave idle.  MACE_OPT_SINGLE_STREAM keeps everything on
// the caller's stream.
constexpr int N_FORK_EVENTS = 8;
struct mace_ctx {
  mace_model_t m;
  double *inv_freq;   // device [head_dim/2]
  hipStream_t side = nullptr;
  hipEvent_t ev_fork[N_FORK_EVENTS] = {}, ev_join = nullptr;
  int n_fork = 0;          // forks issued in the current call
  bool head_two_pass = false;   // MACE_OPT_HEAD_TWO_PASS: every logit of the DPO head from two-term activations
  bool single_stream = false;   // MACE_OPT_SINGLE_STREAM
  int decode_chunk = 0;         // MACE_OPT_DECODE_CHUNK
  std::vector<mace_gemm_plan_t> plan;   // launch decisions of the GEMMs of the last iteration call
  int device = 0;                       // the device that was current in mace_create
  void *static_scratch = nullptr;       // device address of g_static_scratch on that device
  bool prof_on = false;
  unsigned prof_mask = ~0u;        // kernel classes that are timed
  bool prof_open[2] = {false, false};   // per chain: the last mark opened an interval
  std::vector<hipEvent_t> prof_events;
  std::vector<ProfMark> prof_marks;
};

// Scratch of mace_next_token_logits_static: the normalised rows (bf16) of one call.  One copy per GPU,
// held until the process ends; every call on a GPU shares it (overlapping calls race).  Host code
// never uses this name as an address: mace_create asks the runtime for the device address
// (hipGetSymbolAddress, once per handle, with the handle's device current) and keeps it in the context.
constexpr size_t STATIC_SCRATCH_BYTES = (size_t)4 << 20;
static __device__ __align__(256) unsigned char g_static_scratch[STATIC_SCRATCH_BYTES];

namespace {

const char *const PROF_TAGS[] = {"gemm_nt", "gemm_nn", "gemm_tn", "attn_fwd_prefill", "attn_fwd_ft", "attn_decode",
                                 "attn_bwd", "rmsnorm", "rope", "swiglu", "logsoftmax", "dlogits", "misc",
                                 "gemm_nt@side", "gemm_nn@side", "gemm_tn@side"};   // GEMM launches on the side stream
enum { T_GEMM_NT, T_GEMM_NN, T_GEMM_TN, T_ATTN_PREFILL, T_ATTN_FT, T_ATTN_DECODE, T_ATTN_BWD, T_RMSNORM, T_ROPE,
       T_SWIGLU, T_LOGSOFTMAX, T_DLOGITS, T_MISC, T_SIDE0, T_COUNT = T_SIDE0 + 3 };
constexpr size_t PROF_MAX_MARKS = 1 << 15;

void prof_mark(mace_ctx *h, hipStream_t st, int tag, double flops = 0.0, double bytes = 0.0) {
  if (!h->prof_on || h->prof_marks.size() >= h->prof_events.size()) return;
  const int c = h->side && st == h->side ? 1 : 0;
  const bool want = tag >= 0 && ((h->prof_mask >> tag) & 1u);
  if (!want && !h->prof_open[c]) return;           // nothing to open and nothing to close
  if (hipEventRecord(h->prof_events[h->prof_marks.size()], st) != hipSuccess) return;
  h->prof_marks.push_back({want ? tag : -1, c, flops, bytes});
  h->prof_open[c] = want;
}

// Side stream on which work may start once everything issued so far on `st` is done; returns `st`
// itself when the context has no side stream.
hipStream_t side_fork(mace_ctx *h, hipStream_t st) {
  if (!h->side || h->single_stream || h->n_fork >= N_FORK_EVENTS) return st;
  hipEvent_t ev = h->ev_fork[h->n_fork];
  if (hipEventRecord(ev, st) != hipSuccess || hipStreamWaitEvent(h->side, ev, 0) != hipSuccess) return st;
  ++h->n_fork;
  return h->side;
}
// Makes `st` wait for everything issued on the side stream in this call.
hipError_t side_join(mace_ctx *h, hipStream_t st) {
  if (!h->side || h->n_fork == 0) return hipSuccess;
  h->n_fork = 0;
  hipError_t e = hipEventRecord(h->ev_join, h->side);
  if (e != hipSuccess) return e;
  return hipStreamWaitEvent(st, h->ev_join, 0);
}

// Joins the side stream back into the caller's stream on every way out of an iteration call, error
// returns included: work that was forked must not outlive the call (it reads the caller's workspace).
struct SideGuard {
  mace_ctx *h;
  hipStream_t st;
  SideGuard(mace_ctx *h_, hipStream_t st_) : h(h_), st(st_) { (void)side_join(h, st); h->plan.clear(); }
  ~SideGuard() { (void)side_join(h, st); }
};

thread_local std::string g_err;

int fail(int code, const std::string &msg) {
  g_err = msg;
  return code;
}
int hip_fail(hipError_t e, const char *where) {
  return fail(MACE_HIP_ERROR, std::string(where) + ": " + hipGetErrorString(e));
}
#define HIP_TRY(expr, where)                         \
  do {                                               \
    hipError_t e__ = (expr);                         \
    if (e__ != hipSuccess) return hip_fail(e__, where); \
  } while (0)

// Bump allocator over a caller buffer; with base == nullptr it only measures.
struct Bump {
  char *base;
  size_t off = 0;
  explicit Bump(void *b) : base((char *)b) {}
  template <typename T>
  T *take(size_t n) {
    off = align_up(off, 256);
    T *p = base ? (T *)(base + off) : nullptr;
    off += n * sizeof(T);
    return p;
  }
};

struct Dims {
  int d, Hq, Hkv, hd, F, V, qd, kd, nqkv;
  bool bf;
  explicit Dims(const mace_model_t &m)
      : d(m.d_model), Hq(m.n_q_heads), Hkv(m.n_kv_heads), hd(m.head_dim), F(m.d_ff), V(m.vocab),
        qd(m.n_q_heads * m.head_dim), kd(m.n_kv_heads * m.head_dim), nqkv((m.n_q_heads + 2 * m.n_kv_heads) * m.head_dim),
        bf(m.io_dtype == MACE_BF16) {}
};

constexpr int DG_PARTS = 1024;   // blocks (and partial rows) of the RMSNorm backward

// bf16 (hi, lo) views of the seven weight matrices; for bf16 models hi aliases the caller's weights.
struct WSplit {
  const bf16_t *hi[7];
  bf16_t *lo[7];
};
enum { W_Q, W_K, W_V, W_O, W_G, W_U, W_D };

size_t weight_elems(const Dims &D, int i) {
  switch (i) {
    case W_Q: return (size_t)D.qd * D.d;
    case W_K: case W_V: return (size_t)D.kd * D.d;
    case W_O: return (size_t)D.d * D.qd;
    default: return (size_t)D.F * D.d;
  }
}

// Reserve (and for fp32 models fill) the split weights.  need_lo: the forward uses the lo term.
int prepare_weights(const Dims &D, const mace_layer_w_t *w, Bump &ws, bool need_lo, bool run, hipStream_t st, WSplit &out) {
  const void *src[7] = {w ? w->wq : nullptr, w ? w->wk : nullptr, w ? w->wv : nullptr, w ? w->wo : nullptr,
                        w ? w->w_gate : nullptr, w ? w->w_up : nullptr, w ? w->w_down : nullptr};
  for (int i = 0; i < 7; ++i) {
    if (D.bf) {
      out.hi[i] = (const bf16_t *)src[i];
      out.lo[i] = nullptr;
    } else {
      bf16_t *hi = ws.take<bf16_t>(weight_elems(D, i));
      bf16_t *lo = need_lo ? ws.take<bf16_t>(weight_elems(D, i)) : nullptr;
      out.hi[i] = hi;
      out.lo[i] = lo;
      if (run) HIP_TRY(launch_split_f32((const float *)src[i], weight_elems(D, i), hi, lo, st), "split weights");
    }
  }
  return MACE_OK;
}

// ---------------------------------------------------------------- saved activations (ft rows)
struct Saved {
  float *rstd1, *rstd2, *lse, *x1;
  bf16_t *a, *q, *k, *v, *o, *b, *gu;   // gu = [G | U] of the MLP, bf16
  bf16_t *hm;                           // silu(G) * U rounded to bf16: A operand of the down projection, B operand of dWd
  bf16_t *tq, *to;   // adapter variant: scale * (a [A_q;A_k;A_v]^T) [Tf, 3*64] and scale * (o A_o^T) [Tf, 64]
};
constexpr int LR = 64;   // adapter rank as the GEMM sees it (zero-padded)
Saved plan_saved(const Dims &D, size_t Tf, Bump &s) {
  Saved S;
  S.rstd1 = s.take<float>(Tf);
  S.rstd2 = s.take<float>(Tf);
  S.lse = s.take<float>(Tf * D.Hq);
  S.x1 = s.take<float>(Tf * D.d);
  S.gu = s.take<bf16_t>(Tf * 2 * D.F);
  S.hm = s.take<bf16_t>(Tf * D.F);
  S.a = s.take<bf16_t>(Tf * D.d);
  S.q = s.take<bf16_t>(Tf * D.qd);
  S.k = s.take<bf16_t>(Tf * D.kd);
  S.v = s.take<bf16_t>(Tf * D.kd);
  S.o = s.take<bf16_t>(Tf * D.qd);
  S.b = s.take<bf16_t>(Tf * D.d);
  S.tq = s.take<bf16_t>(Tf * 3 * LR);
  S.to = s.take<bf16_t>(Tf * LR);
  return S;
}

// ---------------------------------------------------------------- forward scratch
struct FwdWs {
  // inference rows
  bf16_t *a_i, *q_i, *k_i, *v_i, *o_i, *b_i, *hm_i;
  float *qkv_i, *x1_i, *dec_partial;
  // fine-tune rows
  float *qkv_f;
  bf16_t *a_lo, *q_lo, *k_lo, *v_lo, *o_lo, *b_lo, *hm_lo;
};
FwdWs plan_fwd(const Dims &D, size_t Ti, size_t Tf, int n_decode, int max_ctx, int decode_chunk, Bump &w) {
  FwdWs F;
  F.a_i = w.take<bf16_t>(Ti * D.d);
  F.qkv_i = w.take<float>(Ti * D.nqkv);
  F.q_i = w.take<bf16_t>(Ti * D.qd);
  F.k_i = w.take<bf16_t>(Ti * D.kd);
  F.v_i = w.take<bf16_t>(Ti * D.kd);
  F.o_i = w.take<bf16_t>(Ti * D.qd);
  F.x1_i = w.take<float>(Ti * D.d);
  F.b_i = w.take<bf16_t>(Ti * D.d);
  F.hm_i = w.take<bf16_t>(Ti * D.F);
  F.dec_partial = w.take<float>(decode_partial_floats(n_decode, D.Hq, D.Hkv, D.hd, max_ctx, decode_chunk));
  F.qkv_f = w.take<float>(Tf * D.nqkv);
  F.a_lo = w.take<bf16_t>(Tf * D.d);
  F.q_lo = w.take<bf16_t>(Tf * D.qd);
  F.k_lo = w.take<bf16_t>(Tf * D.kd);
  F.v_lo = w.take<bf16_t>(Tf * D.kd);
  F.o_lo = w.take<bf16_t>(Tf * D.qd);
  F.b_lo = w.take<bf16_t>(Tf * D.d);
  F.hm_lo = w.take<bf16_t>(Tf * D.F);
  return F;
}

// ---------------------------------------------------------------- backward scratch
struct BwdWs {
  bf16_t *dy_bf, *dhm, *dgu, *dx1_bf, *dattn, *dqkv;
  float *db, *dx1, *dvec, *da, *dg_part;
  float2 *cs;      // rotary (cos, sin) of every fine-tune row, [Tf, hd/2]
};
BwdWs plan_bwd(const Dims &D, size_t Tf, Bump &w) {
  BwdWs B;
  B.dy_bf = w.take<bf16_t>(Tf * D.d);
  B.dhm = w.take<bf16_t>(Tf * D.F);
  B.dgu = w.take<bf16_t>(Tf * 2 * D.F);
  B.db = w.take<float>(Tf * D.d);
  B.dx1 = w.take<float>(Tf * D.d);
  B.dx1_bf = w.take<bf16_t>(Tf * D.d);
  B.dattn = w.take<bf16_t>(Tf * D.qd);
  B.dvec = w.take<float>(Tf * D.Hq);
  B.cs = w.take<float2>(Tf * (D.hd / 2));
  B.dqkv = w.take<bf16_t>(Tf * D.nqkv);
  B.da = w.take<float>(Tf * D.d);
  B.dg_part = w.take<float>((size_t)(DG_PARTS + COLSUM_SLICES) * D.d);     // partial rows + scratch of their column sum
  return B;
}

// ---------------------------------------------------------------- adapter (LoRA) scratch

struct LoraWs {
  bf16_t *aqkv_hi, *aqkv_lo;   // [3*LR, d]   rows: A_q | A_k | A_v, each padded to LR rows
  bf16_t *ao_hi, *ao_lo;       // [LR, qd]
  bf16_t *bblk_hi, *bblk_lo;   // [nqkv, 3*LR] block diagonal: B_q | B_k | B_v
  bf16_t *bo_hi, *bo_lo;       // [d, LR]
  float *t_qkv, *t_o;          // forward: u A^T of every row, [rows, 3*LR] and [rows, LR]
  bf16_t *tq_hi, *tq_lo, *to_hi, *to_lo;
  bf16_t *dtq, *dto;           // backward: dy B
  float *dbblk, *dbo, *daqkv, *dao;
};
LoraWs plan_lora(const Dims &D, size_t rows, bool bwd, Bump &w) {
  LoraWs L;
  memset(&L, 0, sizeof(L));
  const bool lo = !D.bf && !bwd;
  L.aqkv_hi = w.take<bf16_t>((size_t)3 * LR * D.d);
  L.ao_hi = w.take<bf16_t>((size_t)LR * D.qd);
  L.bblk_hi = w.take<bf16_t>((size_t)D.nqkv * 3 * LR);
  L.bo_hi = w.take<bf16_t>((size_t)D.d * LR);
  if (lo) {
    L.aqkv_lo = w.take<bf16_t>((size_t)3 * LR * D.d);
    L.ao_lo = w.take<bf16_t>((size_t)LR * D.qd);
    L.bblk_lo = w.take<bf16_t>((size_t)D.nqkv * 3 * LR);
    L.bo_lo = w.take<bf16_t>((size_t)D.d * LR);
  }
  L.tq_hi = w.take<bf16_t>(rows * 3 * LR);
  L.to_hi = w.take<bf16_t>(rows * LR);
  if (!bwd) {
    L.t_qkv = w.take<float>(rows * 3 * LR);
    L.t_o = w.take<float>(rows * LR);
    L.tq_lo = w.take<bf16_t>(rows * 3 * LR);
    L.to_lo = w.take<bf16_t>(rows * LR);
  } else {
    L.dtq = w.take<bf16_t>(rows * 3 * LR);
    L.dto = w.take<bf16_t>(rows * LR);
    L.dbblk = w.take<float>((size_t)D.nqkv * 3 * LR);
    L.dbo = w.take<float>((size_t)D.d * LR);
    L.daqkv = w.take<float>((size_t)3 * LR * D.d);
    L.dao = w.take<float>((size_t)LR * D.qd);
  }
  return L;
}

int check_lora(const mace_lora_t *l) {
  if (!l) return fail(MACE_INVALID_ARG, "lora is null");
  if (!l->a_q || !l->b_q || !l->a_k || !l->b_k || !l->a_v || !l->b_v || !l->a_o || !l->b_o) return fail(MACE_INVALID_ARG, "null adapter pointer");
  if (l->rank < 1 || l->rank > LR) return fail(MACE_BAD_SHAPE, "adapter rank must be in 1..64");
  if (!std::isfinite(l->scale)) return fail(MACE_INVALID_ARG, "adapter scale");
  return MACE_OK;
}

// Pack the caller's adapters into the padded operands.  b_scale multiplies the B matrices (the
// backward folds the adapter scale into them).
int prepare_lora(const Dims &D, const mace_lora_t *l, const LoraWs &L, float b_scale, hipStream_t st) {
  const int r = l->rank;
  {
    const void *src[3] = {l->a_q, l->a_k, l->a_v};
    const int rows[3] = {r, r, r}, cols[3] = {D.d, D.d, D.d}, r0[3] = {0, LR, 2 * LR}, c0[3] = {0, 0, 0};
    HIP_TRY(launch_lora_pack(src, rows, cols, r0, c0, 3, D.bf, 3 * LR, D.d, 1.0f, L.aqkv_hi, L.aqkv_lo, st), "pack A_qkv");
  }
  {
    const void *src[1] = {l->a_o};
    const int rows[1] = {r}, cols[1] = {D.qd}, z[1] = {0};
    HIP_TRY(launch_lora_pack(src, rows, cols, z, z, 1, D.bf, LR, D.qd, 1.0f, L.ao_hi, L.ao_lo, st), "pack A_o");
  }
  {
    const void *src[3] = {l->b_q, l->b_k, l->b_v};
    const int rows[3] = {D.qd, D.kd, D.kd}, cols[3] = {r, r, r}, r0[3] = {0, D.qd, D.qd + D.kd}, c0[3] = {0, LR, 2 * LR};
    HIP_TRY(launch_lora_pack(src, rows, cols, r0, c0, 3, D.bf, D.nqkv, 3 * LR, b_scale, L.bblk_hi, L.bblk_lo, st), "pack B_qkv");
  }
  {
    const void *src[1] = {l->b_o};
    const int rows[1] = {D.d}, cols[1] = {r}, z[1] = {0};
    HIP_TRY(launch_lora_pack(src, rows, cols, z, z, 1, D.bf, D.d, LR, b_scale, L.bo_hi, L.bo_lo, st), "pack B_o");
  }
  return MACE_OK;
}

// ---------------------------------------------------------------- DPO head scratch
struct DpoWs {
  int32_t *row_idx, *label, *seq_id, *partner, *vseq_off, *vprompt;   // the last three: shared-prompt layout only
  bf16_t *n_hi, *n_lo, *dl, *e_hi, *e_lo;
  float *rstd, *logits, *logp_t, *lse, *dlogp, *dn, *dn_part, *dg_part;
};
DpoWs plan_dpo(const Dims &D, size_t R, size_t n_seq, Bump &w) {
  DpoWs P;
  P.row_idx = w.take<int32_t>(R);
  P.label = w.take<int32_t>(R);
  P.seq_id = w.take<int32_t>(R);
  P.partner = w.take<int32_t>(R);
  P.vseq_off = w.take<int32_t>(n_seq + 1);
  P.vprompt = w.take<int32_t>(n_seq);
  P.n_hi = w.take<bf16_t>(R * D.d);
  P.n_lo = w.take<bf16_t>(R * D.d);
  P.rstd = w.take<float>(R);
  P.logits = w.take<float>(R * D.V);
  P.logp_t = w.take<float>(R);
  P.lse = w.take<float>(R);
  P.dlogp = w.take<float>(n_seq);
  P.dl = w.take<bf16_t>(R * D.V);
  P.dn = w.take<float>(R * D.d);
  P.dn_part = w.take<float>(R * D.d * (size_t)(gemm_suggest_k_splits((int)R, D.d, D.V) > 1 ? gemm_suggest_k_splits((int)R, D.d, D.V) : 0));
  P.dg_part = w.take<float>((size_t)(DG_PARTS + COLSUM_SLICES) * D.d);
  if (!D.bf) {
    P.e_hi = w.take<bf16_t>((size_t)D.V * D.d);
    P.e_lo = w.take<bf16_t>((size_t)D.V * D.d);
  } else {
    P.e_hi = P.e_lo = nullptr;
  }
  return P;
}

// ---------------------------------------------------------------- next-token logits scratch
struct LogitWs {
  bf16_t *n_hi, *e_hi;
};
LogitWs plan_logits(const Dims &D, size_t n, Bump &w) {
  LogitWs P;
  P.n_hi = w.take<bf16_t>(n * D.d);
  P.e_hi = D.bf ? nullptr : w.take<bf16_t>((size_t)D.V * D.d);
  return P;
}

int run_gemm(mace_ctx *h, int LA, int LB, GemmParams &p, hipStream_t st, const char *where) {
  if (h->prof_on) {
    double mn = 0.0;
    for (int g = 0; g < p.n_mg; ++g)
      for (int s = 0; s < p.n_ns; ++s) mn += (double)p.mg[g].M * (double)p.ns[s].N;
    prof_mark(h, st, LA == 1 ? T_GEMM_TN : (LB == 1 ? T_GEMM_NN : T_GEMM_NT), 2.0 * mn * (double)p.K);
  }
  const char *why = nullptr;
  hipError_t e = gemm_launch(LA, LB, p, st, &why);
  if (e != hipSuccess) return fail(why ? MACE_BAD_SHAPE : MACE_HIP_ERROR, std::string(where) + ": " + (why ? why : hipGetErrorString(e)));
  if (h->plan.size() < 256) {
    mace_gemm_plan_t r;
    memset(&r, 0, sizeof(r));
    snprintf(r.name, sizeof(r.name), "%s", where);
    r.layout = LA == 1 ? 2 : (LB == 1 ? 1 : 0);
    r.tile_m = p.tile_m; r.tile_n = p.tile_n;
    r.k_splits = p.k_splits > 1 ? p.k_splits : 1;
    r.on_side_stream = h->side && st == h->side ? 1 : 0;
    for (int g = 0; g < p.n_mg; ++g) r.m += p.mg[g].M;
    for (int sg = 0; sg < p.n_ns; ++sg) r.n += p.ns[sg].N;
    r.k = p.K;
    h->plan.push_back(r);
  }
  return MACE_OK;
}
// A weight-gradient GEMM ([M, N] out of K rows) that nothing later in the call depends on: issued on
// the side stream (see mace_ctx) when the products of the main chain around it are small.  Those
// have about (K / 256) x (min(M, N) / 256) output tiles; from two tiles per CU on they fill the chip
// by themselves, and a second resident GEMM only splits the CUs and the L2 between two working
// sets (measured: 2.5 - 3 % slower at 12 K and 64 K rows of a 7B-class layer, 2 % faster at 1.5 K
// and 3.5 K rows).
int run_gemm_side(mace_ctx *h, int LA, int LB, GemmParams &p, hipStream_t st, const char *where) {
  long long M = 0, N = 0;
  for (int g = 0; g < p.n_mg; ++g) M += p.mg[g].M;
  for (int s = 0; s < p.n_ns; ++s) N += p.ns[s].N;
  const bool main_chain_small = (double)p.K * (double)std::min(M, N) < 2.0 * 256 * 65536.0;
  hipStream_t s2 = main_chain_small ? side_fork(h, st) : st;
  const int rc = run_gemm(h, LA, LB, p, s2, where);
  if (rc == MACE_OK && s2 != st) prof_mark(h, s2, -1);
  return rc;
}
#define TRY(expr)                 \
  do {                            \
    int rc__ = (expr);            \
    if (rc__ != MACE_OK) return rc__; \
  } while (0)

GemmParams gp_init(int K, long long lda, long long ldb, long long ldc) {
  GemmParams p;
  memset(&p, 0, sizeof(p));
  p.K = K; p.lda = lda; p.ldb = ldb; p.ldc = ldc; p.ldr = ldc;
  return p;
}
void gp_group(GemmParams &p, const bf16_t *a_hi, const bf16_t *a_lo, void *c, const void *resid, int M, int npass) {
  if (M <= 0) return;
  GemmMGroup &g = p.mg[p.n_mg++];
  g.a[0] = a_hi; g.a[1] = a_lo; g.c = c; g.resid = resid; g.M = M; g.npass = npass;
}
void gp_seg(GemmParams &p, const bf16_t *b_hi, const bf16_t *b_lo, int N, int c_col) {
  GemmNSeg &s = p.ns[p.n_ns++];
  s.b[0] = b_hi; s.b[1] = b_lo; s.N = N; s.c_col = c_col;
}

struct BatchInfo {
  int Tp, Td, Tf, Ti, T, n_seq_all, max_prefill, max_ft, max_ctx;
  double pairs_prefill, pairs_ft;   // sum of L(L+1)/2 (query, key) pairs, for the algorithmic flop counts
  bool prefix;                      // prefill requests attend to cached prefixes through block tables
};

int check_batch(const mace_batch_t *b, BatchInfo &I) {
  if (!b) return fail(MACE_INVALID_ARG, "batch is null");
  if (b->n_prefill < 0 || b->n_decode < 0 || b->n_ft_seq < 0 || b->n_tokens < 0) return fail(MACE_INVALID_ARG, "negative count in batch");
  const int ns = b->n_prefill + b->n_decode + b->n_ft_seq;
  if (!b->seg_offsets_host) return fail(MACE_INVALID_ARG, "seg_offsets_host is null");
  const int32_t *so = b->seg_offsets_host;
  if (so[0] != 0 || so[ns] != b->n_tokens) return fail(MACE_INVALID_ARG, "seg_offsets must start at 0 and end at n_tokens");
  I.max_prefill = I.max_ft = I.max_ctx = 0;
  I.pairs_prefill = I.pairs_ft = 0.0;
  for (int i = 0; i < ns; ++i) {
    const int L = so[i + 1] - so[i];
    if (L < 0) return fail(MACE_INVALID_ARG, "seg_offsets not non-decreasing");
    if (i < b->n_prefill) { I.max_prefill = L > I.max_prefill ? L : I.max_prefill; I.pairs_prefill += 0.5 * L * (L + 1.0); }
    else if (i < b->n_prefill + b->n_decode) { if (L != 1) return fail(MACE_INVALID_ARG, "a decode request must have exactly one row"); }
    else { I.max_ft = L > I.max_ft ? L : I.max_ft; I.pairs_ft += 0.5 * L * (L + 1.0); }
  }
  I.Tp = so[b->n_prefill];
  I.Td = b->n_decode;
  I.Ti = I.Tp + I.Td;
  I.T = b->n_tokens;
  I.Tf = I.T - I.Ti;
  I.n_seq_all = ns;
  if (b->n_tokens > 0 && (!b->seg_offsets || !b->positions)) return fail(MACE_INVALID_ARG, "seg_offsets/positions device pointer is null");
  I.prefix = b->prefill_block_tables || b->prefill_prefix_lens_host || b->prefill_prefix_lens;
  if (I.prefix && b->n_prefill > 0) {
    if (!b->prefill_block_tables || !b->prefill_prefix_lens_host || !b->prefill_prefix_lens || b->max_blocks_per_prefill <= 0)
      return fail(MACE_INVALID_ARG, "prefix sharing needs prefill_block_tables, both prefix length arrays and max_blocks_per_prefill");
    for (int i = 0; i < b->n_prefill; ++i) {
      const int P = b->prefill_prefix_lens_host[i], L = so[i + 1] - so[i];
      if (P < 0) return fail(MACE_INVALID_ARG, "negative prefix length");
      I.pairs_prefill += (double)P * L;
    }
  }
  if ((b->ft_excl_lo == nullptr) != (b->ft_excl_hi == nullptr)) return fail(MACE_INVALID_ARG, "ft_excl_lo and ft_excl_hi go together");
  if (b->n_decode > 0) {
    if (!b->context_lens_host || !b->context_lens || !b->block_tables) return fail(MACE_INVALID_ARG, "decode descriptors are null");
    for (int i = 0; i < b->n_decode; ++i) {
      const int n = b->context_lens_host[i];
      if (n < 0) return fail(MACE_INVALID_ARG, "negative context length");
      I.max_ctx = n > I.max_ctx ? n : I.max_ctx;
    }
  }
  return MACE_OK;
}

}  // namespace

extern "C" {

const char *mace_last_error(void) { return g_err.c_str(); }

int mace_create(mace_handle_t *out, const mace_model_t *model) {
  if (!out || !model) return fail(MACE_INVALID_ARG, "mace_create: null argument");
  const mace_model_t &m = *model;
  if (m.d_model <= 0 || m.n_q_heads <= 0 || m.n_kv_heads <= 0 || m.d_ff <= 0 || m.vocab <= 0) return fail(MACE_BAD_SHAPE, "non-positive dimension");
  if (m.head_dim != 64 && m.head_dim != 128) return fail(MACE_BAD_SHAPE, "head_dim must be 64 or 128");
  if (m.n_q_heads % m.n_kv_heads) return fail(MACE_BAD_SHAPE, "n_q_heads must be a multiple of n_kv_heads");
  const int grp = m.n_q_heads / m.n_kv_heads;
  if (grp != 1 && grp != 2 && grp != 4 && grp != 8) return fail(MACE_BAD_SHAPE, "n_q_heads / n_kv_heads must be 1, 2, 4 or 8");
  if (m.d_model % 64 || m.d_ff % 64 || m.vocab % 64) return fail(MACE_BAD_SHAPE, "d_model, d_ff and vocab must be multiples of 64");
  if (m.d_model > 8192) return fail(MACE_BAD_SHAPE, "d_model must not exceed 8192");
  if (m.io_dtype != MACE_F32 && m.io_dtype != MACE_BF16) return fail(MACE_INVALID_ARG, "io_dtype");
  if (!(m.rms_eps >= 0.f) || !(m.rope_theta > 0.f)) return fail(MACE_INVALID_ARG, "rms_eps / rope_theta");
  mace_ctx *c = new (std::nothrow) mace_ctx;
  if (!c) return fail(MACE_HIP_ERROR, "out of host memory");
  c->m = m;
  c->inv_freq = nullptr;
  const int half = m.head_dim / 2;
  std::vector<double> f(half);
  for (int i = 0; i < half; ++i) f[i] = std::pow((double)m.rope_theta, -2.0 * i / m.head_dim);
  hipError_t e = hipMalloc((void **)&c->inv_freq, half * sizeof(double));
  if (e == hipSuccess) e = hipMemcpy(c->inv_freq, f.data(), half * sizeof(double), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    if (c->inv_freq) (void)hipFree(c->inv_freq);
    delete c;
    return hip_fail(e, "mace_create");
  }
  e = hipGetDevice(&c->device);
  if (e == hipSuccess) e = hipGetSymbolAddress(&c->static_scratch, HIP_SYMBOL(g_static_scratch));
  if (e != hipSuccess || !c->static_scratch) {
    mace_destroy(c);
    return e != hipSuccess ? hip_fail(e, "mace_create: static scratch address") : fail(MACE_HIP_ERROR, "mace_create: static scratch address is null");
  }
  e = hipStreamCreateWithFlags(&c->side, hipStreamNonBlocking);
  for (int i = 0; i < N_FORK_EVENTS && e == hipSuccess; ++i) e = hipEventCreateWithFlags(&c->ev_fork[i], hipEventDisableTiming);
  if (e == hipSuccess) e = hipEventCreateWithFlags(&c->ev_join, hipEventDisableTiming);
  if (e != hipSuccess) {
    mace_destroy(c);
    return hip_fail(e, "mace_create: side stream");
  }
  *out = c;
  return MACE_OK;
}

int mace_set_option(mace_handle_t h, int32_t option, int32_t value) {
  if (!h) return fail(MACE_INVALID_ARG, "handle is null");
  switch (option) {
    case MACE_OPT_HEAD_TWO_PASS:
      if (value != 0 && value != 1) return fail(MACE_INVALID_ARG, "MACE_OPT_HEAD_TWO_PASS takes 0 or 1");
      h->head_two_pass = value != 0;
      return MACE_OK;
    case MACE_OPT_SINGLE_STREAM:
      if (value != 0 && value != 1) return fail(MACE_INVALID_ARG, "MACE_OPT_SINGLE_STREAM takes 0 or 1");
      h->single_stream = value != 0;
      return MACE_OK;
    case MACE_OPT_DECODE_CHUNK:
      if (value != 0 && (value < 512 || value > 4096 || (value & (value - 1)))) return fail(MACE_INVALID_ARG, "MACE_OPT_DECODE_CHUNK takes 0 or a power of two in 512..4096");
      h->decode_chunk = value;
      return MACE_OK;
    default:
      return fail(MACE_INVALID_ARG, "unknown option");
  }
}

int mace_launch_plan(mace_handle_t h, mace_gemm_plan_t *out, int32_t max_entries, int32_t *n_out) {
  if (!h || !n_out || max_entries < 0 || (max_entries > 0 && !out)) return fail(MACE_INVALID_ARG, "mace_launch_plan: bad argument");
  const int32_t n = (int32_t)std::min<size_t>(h->plan.size(), (size_t)max_entries);
  for (int32_t i = 0; i < n; ++i) out[i] = h->plan[i];
  *n_out = (int32_t)h->plan.size();
  return MACE_OK;
}

int mace_gemm_bf16(mace_handle_t h, const mace_gemm_desc_t *d, void *stream) {
  if (!h || !d || !d->a || !d->b || !d->c) return fail(MACE_INVALID_ARG, "mace_gemm_bf16: null argument");
  if (d->M <= 0 || d->N <= 0 || d->K <= 0) return fail(MACE_BAD_SHAPE, "mace_gemm_bf16: M, N and K must be positive");
  if (d->swiglu == 1 && !d->b_up) return fail(MACE_INVALID_ARG, "mace_gemm_bf16: SwiGLU mode needs b_up");
  if (d->swiglu == 2 && (!d->c_gu || d->kernel != 1)) return fail(MACE_INVALID_ARG, "mace_gemm_bf16: SwiGLU backward mode needs c_gu and kernel = 1");
  GemmParams p = gp_init(d->K, d->lda, d->ldb, d->ldc);
  p.ldr = d->ldr;
  p.out_bf16 = d->swiglu ? 1 : d->out_bf16;
  p.swiglu_bwd = d->swiglu == 2;
  p.resid_kind = d->resid ? d->resid_kind : 0;
  p.force_w4 = d->kernel == 1;
  gp_group(p, (const bf16_t *)d->a, (const bf16_t *)d->a_lo, d->c, d->resid, d->M, d->a_lo ? 2 : 1);
  p.mg[0].c_lo = d->swiglu ? d->c_lo : nullptr;
  p.mg[0].c_gu = d->swiglu ? d->c_gu : nullptr;
  gp_seg(p, (const bf16_t *)d->b, nullptr, d->N, 0);
  if (d->swiglu == 1) {
    p.swiglu = 1;
    gp_seg(p, (const bf16_t *)d->b_up, nullptr, d->N, 0);
  }
  if (d->rope_cs) {
    if (d->swiglu || d->kernel != 1 || d->resid) return fail(MACE_INVALID_ARG, "mace_gemm_bf16: the rotary form takes kernel = 1 and neither SwiGLU mode nor a residual");
    p.out_bf16 = 0;
    p.mg[0].rope = 1;
    p.rope_cs = d->rope_cs;
    p.ns[0].rope_hi = d->c; p.ns[0].rope_lo = d->c_lo; p.ns[0].rope_rot = d->rope_rotate ? 1 : 0;
  }
  h->plan.clear();
  return run_gemm(h, d->layout_a, d->layout_b, p, (hipStream_t)stream, "mace_gemm_bf16");
}

void mace_destroy(mace_handle_t h) {
  if (!h) return;
  if (h->inv_freq) (void)hipFree(h->inv_freq);
  if (h->side) {
    (void)hipStreamSynchronize(h->side);
    (void)hipStreamDestroy(h->side);
  }
  for (hipEvent_t e : h->ev_fork)
    if (e) (void)hipEventDestroy(e);
  if (h->ev_join) (void)hipEventDestroy(h->ev_join);
  for (hipEvent_t e : h->prof_events) (void)hipEventDestroy(e);
  delete h;
}

int mace_profile_enable(mace_handle_t h, int on) {
  if (!h) return fail(MACE_INVALID_ARG, "handle is null");
  h->prof_marks.clear();
  h->prof_open[0] = h->prof_open[1] = false;
  h->prof_mask = on == 1 ? ~0u : (unsigned)on >> 1;
  if (on && h->prof_events.empty()) {
    h->prof_events.reserve(PROF_MAX_MARKS);
    for (size_t i = 0; i < PROF_MAX_MARKS; ++i) {
      hipEvent_t e;
      HIP_TRY(hipEventCreate(&e), "hipEventCreate");
      h->prof_events.push_back(e);
    }
  }
  h->prof_on = on != 0;
  return MACE_OK;
}

int mace_profile_collect(mace_handle_t h, mace_profile_entry_t *out, int32_t max_entries, int32_t *n_out) {
  if (!h || !out || !n_out || max_entries < T_COUNT) return fail(MACE_INVALID_ARG, "mace_profile_collect: bad argument");
  const size_t n = h->prof_marks.size();
  if (n) HIP_TRY(hipEventSynchronize(h->prof_events[n - 1]), "hipEventSynchronize");
  for (int t = 0; t < T_COUNT; ++t) {
    memset(&out[t], 0, sizeof(out[t]));
    snprintf(out[t].name, sizeof(out[t].name), "%s", PROF_TAGS[t]);
  }
  if (h->side) HIP_TRY(hipStreamSynchronize(h->side), "hipStreamSynchronize");
  long prev[2] = {-1, -1};                       // previous mark of each chain
  for (size_t i = 0; i < n; ++i) {
    const int c = h->prof_marks[i].chain;
    if (prev[c] >= 0 && h->prof_marks[prev[c]].tag >= 0) {
      const ProfMark &m = h->prof_marks[prev[c]];
      float ms = 0.f;
      HIP_TRY(hipEventElapsedTime(&ms, h->prof_events[prev[c]], h->prof_events[i]), "hipEventElapsedTime");
      const int tg = c == 1 && m.tag <= T_GEMM_TN ? T_SIDE0 + m.tag : m.tag;   // side-stream GEMMs are classes of their own
      out[tg].launches += 1;
      out[tg].side_launches += c;
      out[tg].ms += ms;
      out[tg].flops += m.flops;
      out[tg].bytes += m.bytes;
    }
    prev[c] = (long)i;
  }
  *n_out = T_COUNT;
  h->prof_marks.clear();
  h->prof_open[0] = h->prof_open[1] = false;
  return MACE_OK;
}

size_t mace_fwd_saved_bytes(mace_handle_t h, int32_t n_ft_tokens) {
  if (!h || n_ft_tokens < 0) return 0;
  Bump b(nullptr);
  plan_saved(Dims(h->m), (size_t)n_ft_tokens, b);
  return align_up(b.off, 256);
}

size_t mace_workspace_bytes(mace_handle_t h, int32_t n_tokens, int32_t n_ft_tokens, int32_t n_decode,
                            int32_t max_context, int32_t n_loss_rows) {
  if (!h || n_tokens < 0 || n_ft_tokens < 0 || n_ft_tokens > n_tokens || n_decode < 0 || max_context < 0 || n_loss_rows < 0) return 0;
  const Dims D(h->m);
  WSplit ws;
  Bump f(nullptr), b(nullptr), p(nullptr);
  prepare_weights(D, nullptr, f, true, false, nullptr, ws);
  plan_fwd(D, (size_t)(n_tokens - n_ft_tokens), (size_t)n_ft_tokens, n_decode, max_context, h->decode_chunk, f);
  plan_lora(D, (size_t)n_tokens, false, f);
  prepare_weights(D, nullptr, b, false, false, nullptr, ws);
  plan_bwd(D, (size_t)n_ft_tokens, b);
  plan_lora(D, (size_t)n_ft_tokens, true, b);
  plan_dpo(D, (size_t)n_loss_rows, 1u << 16, p);
  Bump lg(nullptr);
  plan_logits(D, (size_t)(n_tokens - n_ft_tokens), lg);
  size_t m = f.off > b.off ? f.off : b.off;
  m = m > p.off ? m : p.off;
  m = m > lg.off ? m : lg.off;
  return align_up(m, 256) + 256;
}

static int next_token_logits_impl(mace_handle_t h, const float *y, const int32_t *row_idx, int32_t n, const void *g_final, const void *w_lm,
                                  float *logits_out, int32_t *next_token, void *workspace, size_t workspace_bytes, void *stream) {
  const Dims D(h->m);
  hipStream_t st = (hipStream_t)stream;
  h->plan.clear();
  Bump wsb(workspace);
  LogitWs P = plan_logits(D, (size_t)n, wsb);
  if (wsb.off > workspace_bytes) return fail(MACE_WORKSPACE_TOO_SMALL, "next-token workspace too small");
  const bf16_t *e_hi = (const bf16_t *)w_lm;
  if (!D.bf) {
    prof_mark(h, st, T_MISC);
    HIP_TRY(launch_split_f32((const float *)w_lm, (size_t)D.V * D.d, P.e_hi, nullptr, st), "split E");
    e_hi = P.e_hi;
  }
  prof_mark(h, st, T_RMSNORM);
  HIP_TRY(launch_rmsnorm_fwd(y, false, row_idx, g_final, D.bf, n, D.d, h->m.rms_eps, P.n_hi, nullptr, nullptr, st), "final rmsnorm");
  {
    GemmParams p = gp_init(D.d, D.d, D.d, D.V);
    gp_group(p, P.n_hi, nullptr, logits_out, nullptr, n, 1);
    gp_seg(p, e_hi, nullptr, D.V, 0);
    TRY(run_gemm(h, 0, 0, p, st, "next-token logits gemm"));
  }
  if (next_token) {
    prof_mark(h, st, T_MISC);
    HIP_TRY(launch_argmax_rows(logits_out, n, D.V, next_token, st), "argmax");
  }
  prof_mark(h, st, -1);
  return MACE_OK;
}

int mace_next_token_logits(mace_handle_t h, const float *y, const int32_t *row_idx, int32_t n, const void *g_final, const void *w_lm,
                           float *logits_out, int32_t *next_token, void *workspace, size_t workspace_bytes, void *stream) {
  if (!h || !y || !g_final || !w_lm || !logits_out || n < 0) return fail(MACE_INVALID_ARG, "mace_next_token_logits: bad argument");
  if (n == 0) return MACE_OK;
  if (!workspace || ((uintptr_t)workspace & 255)) return fail(MACE_INVALID_ARG, "workspace must be non-null and 256-byte aligned");
  return next_token_logits_impl(h, y, row_idx, n, g_final, w_lm, logits_out, next_token, workspace, workspace_bytes, stream);
}

int mace_next_token_logits_static(mace_handle_t h, const float *y, const int32_t *row_idx, int32_t n, const void *g_final,
                                  const void *w_lm, float *logits_out, int32_t *next_token, void *stream) {
  if (!h || !y || !g_final || !w_lm || !logits_out || n < 0) return fail(MACE_INVALID_ARG, "mace_next_token_logits_static: bad argument");
  if (n == 0) return MACE_OK;
  const Dims D(h->m);
  if (!D.bf) return fail(MACE_BAD_SHAPE, "mace_next_token_logits_static needs a bf16 model (fp32 weights would need a converted copy of the head)");
  {
    Bump m(nullptr);
    plan_logits(D, (size_t)n, m);
    if (m.off > STATIC_SCRATCH_BYTES) {
      char msg[160];
      snprintf(msg, sizeof(msg), "mace_next_token_logits_static: %d rows of d_model %d need %zu bytes of scratch, the built-in buffer holds %zu",
               n, D.d, m.off, STATIC_SCRATCH_BYTES);
      return fail(MACE_WORKSPACE_TOO_SMALL, msg);
    }
  }
  int dev = -1;
  HIP_TRY(hipGetDevice(&dev), "hipGetDevice");
  if (dev != h->device) return fail(MACE_INVALID_ARG, "mace_next_token_logits_static: the handle was created on another device than the current one");
  return next_token_logits_impl(h, y, row_idx, n, g_final, w_lm, logits_out, next_token, h->static_scratch, STATIC_SCRATCH_BYTES, stream);
}

int mace_adamw_step(mace_handle_t h, void *param, float *master, const float *grad, float *m, float *v, int64_t n, float lr,
                    float beta1, float beta2, float eps, float weight_decay, int32_t step, void *stream) {
  if (!h || !param || !grad || !m || !v || n < 0) return fail(MACE_INVALID_ARG, "mace_adamw_step: bad argument");
  if (step < 1) return fail(MACE_INVALID_ARG, "step counts from 1");
  if (!(beta1 >= 0.f && beta1 < 1.f) || !(beta2 >= 0.f && beta2 < 1.f) || !(eps >= 0.f) || !std::isfinite(lr) || !std::isfinite(weight_decay))
    return fail(MACE_INVALID_ARG, "AdamW hyper-parameters");
  const double c1 = 1.0 / (1.0 - std::pow((double)beta1, (double)step)), c2 = 1.0 / (1.0 - std::pow((double)beta2, (double)step));
  HIP_TRY(launch_adamw(param, h->m.io_dtype == MACE_BF16, master, grad, m, v, (size_t)n, lr, beta1, beta2, eps, weight_decay, (float)c1, (float)c2,
                       (hipStream_t)stream), "adamw");
  return MACE_OK;
}

int mace_head_norm_stats(mace_handle_t h, const float *norms, const int32_t *t_count, int32_t n, int32_t n_heads, float *abar,
                         int32_t *last_used, int32_t window, float tau, int32_t *prune, void *stream) {
  if (!h || !norms || !t_count || !abar || n < 0 || n_heads <= 0) return fail(MACE_INVALID_ARG, "mace_head_norm_stats: bad argument");
  if ((last_used == nullptr) != (prune == nullptr)) return fail(MACE_INVALID_ARG, "last_used and prune go together");
  if ((long long)n * n_heads > (1ll << 30)) return fail(MACE_BAD_SHAPE, "too many (request, head) pairs");
  if (prune && (window < 0 || !(tau >= 0.f))) return fail(MACE_INVALID_ARG, "window / tau");
  HIP_TRY(launch_head_norm_stats(norms, t_count, n, n_heads, abar, last_used, window, tau, prune, (hipStream_t)stream), "head norm stats");
  return MACE_OK;
}

int mace_kv_head_budget(const double *abar, int32_t n_heads, int64_t c_total, int64_t *c_out) {
  if (!abar || !c_out || n_heads <= 0 || c_total < 0) return fail(MACE_INVALID_ARG, "mace_kv_head_budget: bad argument");
  double sum = 0.0;
  for (int i = 0; i < n_heads; ++i) {
    if (!(abar[i] > 0.0) || !std::isfinite(abar[i])) return fail(MACE_INVALID_ARG, "head norms must be positive and finite");
    sum += abar[i];
  }
  std::vector<double> w(n_heads);
  int64_t used = 0;
  for (int i = 0; i < n_heads; ++i) {
    w[i] = abar[i] / sum;
    c_out[i] = (int64_t)std::floor(w[i] * (double)c_total);
    used += c_out[i];
  }
  std::vector<int> order(n_heads);
  for (int i = 0; i < n_heads; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return w[a] > w[b]; });
  int64_t left = c_total - used;
  for (int i = 0; i < n_heads && left > 0; ++i, --left) c_out[order[i]] += 1;
  return MACE_OK;
}

int mace_kv_slot_mapping(const int32_t *block_table, int32_t table_len, int32_t block_size, int32_t start_pos, int32_t n,
                         int32_t *slots_out) {
  if (!block_table || !slots_out || table_len < 0 || start_pos < 0 || n < 0) return fail(MACE_INVALID_ARG, "mace_kv_slot_mapping: bad argument");
  if (block_size <= 0 || (block_size & (block_size - 1))) return fail(MACE_INVALID_ARG, "block_size must be a power of two");
  for (int32_t i = 0; i < n; ++i) {
    const int64_t p = (int64_t)start_pos + i;
    const int64_t bi = p / block_size;
    if (bi >= table_len) return fail(MACE_INVALID_ARG, "position beyond the block table");
    const int64_t blk = block_table[bi];
    if (blk < 0) return fail(MACE_INVALID_ARG, "negative block id");
    const int64_t slot = blk * block_size + p % block_size;
    if (slot > INT32_MAX) return fail(MACE_INVALID_ARG, "slot does not fit int32");
    slots_out[i] = (int32_t)slot;
  }
  return MACE_OK;
}

static int check_cache(const mace_kv_cache_t *c) {
  if (!c || !c->k || !c->v) return fail(MACE_INVALID_ARG, "kv cache is null");
  if (c->num_blocks <= 0) return fail(MACE_INVALID_ARG, "kv cache has no blocks");
  if (c->block_size <= 0 || c->block_size > 256 || (c->block_size & (c->block_size - 1))) return fail(MACE_INVALID_ARG, "block_size must be a power of two in 1..256");
  return MACE_OK;
}

int mace_kv_cache_append(mace_handle_t h, mace_kv_cache_t *cache, const void *k_new, const void *v_new,
                         const int32_t *slot_mapping, int32_t n, void *stream) {
  if (!h) return fail(MACE_INVALID_ARG, "handle is null");
  TRY(check_cache(cache));
  if (n < 0 || (n > 0 && (!k_new || !v_new || !slot_mapping))) return fail(MACE_INVALID_ARG, "mace_kv_cache_append: bad argument");
  const Dims D(h->m);
  prof_mark(h, (hipStream_t)stream, T_MISC);
  HIP_TRY(launch_kv_append(cache->k, cache->v, D.bf, cache->num_blocks * cache->block_size, cache->block_size, D.Hkv, D.hd, k_new, v_new, slot_mapping, n, (hipStream_t)stream), "kv append");
  return MACE_OK;
}

int mace_kv_cache_gather(mace_handle_t h, const mace_kv_cache_t *cache, const int32_t *block_table, int32_t ctx_len,
                         void *k_out, void *v_out, int64_t *slots_out, void *stream) {
  if (!h) return fail(MACE_INVALID_ARG, "handle is null");
  TRY(check_cache(cache));
  if (ctx_len < 0 || (ctx_len > 0 && (!block_table || !k_out || !v_out))) return fail(MACE_INVALID_ARG, "mace_kv_cache_gather: bad argument");
  const Dims D(h->m);
  prof_mark(h, (hipStream_t)stream, T_MISC);
  HIP_TRY(launch_kv_gather(cache->k, cache->v, D.bf, cache->num_blocks, cache->block_size, D.Hkv, D.hd, block_table, ctx_len, k_out, v_out, (long long *)slots_out, (hipStream_t)stream), "kv gather");
  return MACE_OK;
}

static int layer_fwd_impl(mace_handle_t h, const mace_layer_w_t *w, const mace_lora_t *lora, const mace_batch_t *batch,
                          mace_kv_cache_t *cache, const void *x, float *y, void *saved, void *workspace,
                          size_t workspace_bytes, void *stream) {
  if (!h || !w || !x || !y) return fail(MACE_INVALID_ARG, "mace_hybrid_layer_fwd: null argument");
  if (lora) TRY(check_lora(lora));
  if (!w->g_attn || !w->wq || !w->wk || !w->wv || !w->wo || !w->g_mlp || !w->w_gate || !w->w_up || !w->w_down) return fail(MACE_INVALID_ARG, "null weight pointer");
  BatchInfo I;
  TRY(check_batch(batch, I));
  const Dims D(h->m);
  hipStream_t st = (hipStream_t)stream;
  if (I.T == 0) return MACE_OK;
  if (I.Ti > 0) {
    TRY(check_cache(cache));
    if (!batch->slot_mapping) return fail(MACE_INVALID_ARG, "slot_mapping is null");
    if (I.Td > 0) {
      if (batch->max_blocks_per_req <= 0) return fail(MACE_INVALID_ARG, "max_blocks_per_req");
      if ((long long)I.max_ctx + 1 > (long long)batch->max_blocks_per_req * cache->block_size) return fail(MACE_INVALID_ARG, "context longer than the block table");
    }
  }
  if (I.prefix && batch->n_prefill > 0) {
    if (!D.bf) return fail(MACE_BAD_SHAPE, "prefix sharing needs a bf16 cache");
    for (int i = 0; i < batch->n_prefill; ++i) {
      const long long need = (long long)batch->prefill_prefix_lens_host[i] + batch->seg_offsets_host[i + 1] - batch->seg_offsets_host[i];
      if (need > (long long)batch->max_blocks_per_prefill * cache->block_size) return fail(MACE_INVALID_ARG, "prefix + new tokens longer than the prefill block table");
    }
  }
  if (I.Tf > 0 && !saved) return fail(MACE_INVALID_ARG, "saved is null");
  if (!workspace) return fail(MACE_INVALID_ARG, "workspace is null");
  if (((uintptr_t)workspace & 255) || ((uintptr_t)saved & 255)) return fail(MACE_INVALID_ARG, "workspace/saved must be 256-byte aligned");

  // layout (measure first, then bind)
  WSplit W;
  {
    Bump m(nullptr);
    WSplit tmp;
    prepare_weights(D, w, m, true, false, st, tmp);
    plan_fwd(D, I.Ti, I.Tf, I.Td, I.max_ctx, h->decode_chunk, m);
    if (lora) plan_lora(D, (size_t)I.T, false, m);
    if (m.off > workspace_bytes) return fail(MACE_WORKSPACE_TOO_SMALL, "forward workspace too small");
  }
  SideGuard side_guard(h, st);      // waits for side-stream work an earlier failed call may have left; joins on every return
  Bump wsb(workspace), svb(saved);
  TRY(prepare_weights(D, w, wsb, true, true, st, W));
  FwdWs F = plan_fwd(D, I.Ti, I.Tf, I.Td, I.max_ctx, h->decode_chunk, wsb);
  LoraWs L;
  if (lora) {
    L = plan_lora(D, (size_t)I.T, false, wsb);
    prof_mark(h, st, T_MISC);
    TRY(prepare_lora(D, lora, L, 1.0f, st));
  }
  Saved S = plan_saved(D, I.Tf, svb);
  const int np_ft = D.bf ? 2 : 3;
  const size_t es = D.bf ? 2 : 4;
  const char *xb = (const char *)x;
  const int resid_x = D.bf ? 2 : 1;

  // 1. RMSNorm (attention)
  prof_mark(h, st, T_RMSNORM);
  HIP_TRY(launch_rmsnorm_fwd(x, D.bf, nullptr, w->g_attn, D.bf, I.Ti, D.d, h->m.rms_eps, F.a_i, nullptr, nullptr, st), "rmsnorm1");
  prof_mark(h, st, T_RMSNORM);
  HIP_TRY(launch_rmsnorm_fwd(xb + (size_t)I.Ti * D.d * es, D.bf, nullptr, w->g_attn, D.bf, I.Tf, D.d, h->m.rms_eps, S.a, F.a_lo, S.rstd1, st), "rmsnorm1 ft");
  // 2. QKV projection, all rows in one launch.  Adapter variant: t = a [A_q; A_k; A_v]^T is a skinny
  // product that runs beside the main one on the side stream; then qkv += (scale t) blockdiag(B)^T.
  if (lora) {
    hipStream_t s2 = side_fork(h, st);
    GemmParams p = gp_init(D.d, D.d, D.d, 3 * LR);
    gp_group(p, S.a, F.a_lo, L.t_qkv + (size_t)I.Ti * 3 * LR, nullptr, I.Tf, np_ft);
    gp_group(p, F.a_i, nullptr, L.t_qkv, nullptr, I.Ti, 1);
    gp_seg(p, L.aqkv_hi, L.aqkv_lo, 3 * LR, 0);
    TRY(run_gemm(h, 0, 0, p, s2, "lora t_qkv gemm"));
    prof_mark(h, s2, T_MISC);
    HIP_TRY(launch_scale_split(L.t_qkv, (size_t)I.Ti * 3 * LR, lora->scale, L.tq_hi, nullptr, s2), "lora t_qkv split");
    HIP_TRY(launch_scale_split(L.t_qkv + (size_t)I.Ti * 3 * LR, (size_t)I.Tf * 3 * LR, lora->scale, S.tq, L.tq_lo, s2), "lora t_qkv split ft");
    if (s2 != st) prof_mark(h, s2, -1);
  }
  // Where the product runs on the four-wave kernel (and no adapter correction has to be added to it first), the
  // rotary embedding and the operand split of the fine-tune rows happen in its epilogue: those rows of qkv never
  // exist in fp32, and their angle table takes the place of the fp32 buffer.
  bool rope_fused = false;
  {
    GemmParams p = gp_init(D.d, D.d, D.d, D.nqkv);
    gp_group(p, S.a, F.a_lo, F.qkv_f, nullptr, I.Tf, np_ft);
    gp_group(p, F.a_i, nullptr, F.qkv_i, nullptr, I.Ti, 1);
    gp_seg(p, W.hi[W_Q], W.lo[W_Q], D.qd, 0);
    gp_seg(p, W.hi[W_K], W.lo[W_K], D.kd, D.qd);
    gp_seg(p, W.hi[W_V], W.lo[W_V], D.kd, D.qd + D.kd);
    if (!lora && D.hd == 128 && I.Tf > 0) {
      GemmParams pr = p;
      pr.mg[0].rope = 1;
      pr.rope_cs = F.qkv_f;
      pr.ns[0].rope_hi = S.q; pr.ns[0].rope_lo = F.q_lo; pr.ns[0].rope_rot = 1;
      pr.ns[1].rope_hi = S.k; pr.ns[1].rope_lo = F.k_lo; pr.ns[1].rope_rot = 1;
      pr.ns[2].rope_hi = S.v; pr.ns[2].rope_lo = F.v_lo; pr.ns[2].rope_rot = 0;
      if (gemm_uses_four_wave(0, 0, pr)) {
        prof_mark(h, st, T_ROPE);
        HIP_TRY(launch_rope_table(batch->positions + I.Ti, h->inv_freq, I.Tf, D.hd, (float2 *)F.qkv_f, st), "rope table");
        TRY(run_gemm(h, 0, 0, pr, st, "qkv gemm + rope"));
        rope_fused = true;
      }
    }
    if (!rope_fused) TRY(run_gemm(h, 0, 0, p, st, "qkv gemm"));
  }
  if (lora) {
    HIP_TRY(side_join(h, st), "join side stream");
    GemmParams p2 = gp_init(3 * LR, 3 * LR, 3 * LR, D.nqkv);
    p2.resid_kind = 1; p2.ldr = D.nqkv;
    gp_group(p2, S.tq, L.tq_lo, F.qkv_f, F.qkv_f, I.Tf, np_ft);
    gp_group(p2, L.tq_hi, nullptr, F.qkv_i, F.qkv_i, I.Ti, 1);
    gp_seg(p2, L.bblk_hi, L.bblk_lo, D.nqkv, 0);
    TRY(run_gemm(h, 0, 0, p2, st, "lora qkv gemm"));
  }
  // 3. RoPE, operand split, KV append of the inference rows
  if (I.Ti > 0) {
    prof_mark(h, st, T_ROPE);
    HIP_TRY(launch_rope_split(F.qkv_i, batch->positions, h->inv_freq, I.Ti, D.Hq, D.Hkv, D.hd, F.q_i, F.k_i, F.v_i, nullptr, nullptr, nullptr,
                              batch->slot_mapping, cache->k, cache->v, D.bf, cache->num_blocks * cache->block_size, cache->block_size, st), "rope");
  }
  if (!rope_fused) {
    prof_mark(h, st, T_ROPE);
    HIP_TRY(launch_rope_split(F.qkv_f, batch->positions + I.Ti, h->inv_freq, I.Tf, D.Hq, D.Hkv, D.hd, S.q, S.k, S.v, F.q_lo, F.k_lo, F.v_lo,
                              nullptr, nullptr, nullptr, D.bf, 0, 1, st), "rope ft");
  }
  // 4. attention: prefill (causal), decode (paged), fine-tune (causal, split operands, LSE kept)
  prof_mark(h, st, T_ATTN_PREFILL, 4.0 * D.hd * D.Hq * I.pairs_prefill);
  if (I.prefix && batch->n_prefill > 0)
    HIP_TRY(launch_attn_fwd_paged(F.q_i, cache->k, cache->v, cache->num_blocks, cache->block_size, batch->prefill_block_tables, batch->max_blocks_per_prefill,
                                  batch->prefill_prefix_lens, batch->seg_offsets, 0, batch->n_prefill, I.max_prefill, D.Hq, D.Hkv, D.hd, F.o_i, st), "prefix-shared prefill attention");
  else
    HIP_TRY(launch_attn_fwd(F.q_i, F.k_i, F.v_i, nullptr, nullptr, nullptr, batch->seg_offsets, 0, batch->n_prefill, I.max_prefill, D.Hq, D.Hkv, D.hd, F.o_i, nullptr, nullptr, st), "prefill attention");
  if (I.Td > 0) {
    double kv_tokens = 0.0;
    for (int i = 0; i < I.Td; ++i) kv_tokens += (double)batch->context_lens_host[i] + 1.0;
    prof_mark(h, st, T_ATTN_DECODE, 4.0 * kv_tokens * D.Hq * D.hd, kv_tokens * 2.0 * D.Hkv * D.hd * (D.bf ? 2.0 : 4.0));
    HIP_TRY(launch_attn_decode(F.q_i + (size_t)I.Tp * D.qd, cache->k, cache->v, D.bf, cache->num_blocks, cache->block_size, batch->block_tables, batch->max_blocks_per_req,
                               batch->context_lens, I.Td, I.max_ctx, D.Hq, D.Hkv, D.hd, F.dec_partial, F.o_i + (size_t)I.Tp * D.qd, batch->decode_head_norms, st, h->decode_chunk), "decode attention");
  }
  prof_mark(h, st, T_ATTN_FT, 4.0 * D.hd * D.Hq * I.pairs_ft);
  HIP_TRY(launch_attn_fwd(S.q, S.k, S.v, F.q_lo, F.k_lo, F.v_lo, batch->seg_offsets + batch->n_prefill + batch->n_decode, I.Ti, batch->n_ft_seq, I.max_ft, D.Hq, D.Hkv, D.hd, S.o, F.o_lo, S.lse, st, batch->ft_excl_lo, batch->ft_excl_hi), "ft attention");
  // 5. output projection + residual (adapter variant: t = o A_o^T beside it, then x1 += (scale t) B_o^T)
  if (lora) {
    hipStream_t s2 = side_fork(h, st);
    GemmParams p = gp_init(D.qd, D.qd, D.qd, LR);
    gp_group(p, S.o, F.o_lo, L.t_o + (size_t)I.Ti * LR, nullptr, I.Tf, np_ft);
    gp_group(p, F.o_i, nullptr, L.t_o, nullptr, I.Ti, 1);
    gp_seg(p, L.ao_hi, L.ao_lo, LR, 0);
    TRY(run_gemm(h, 0, 0, p, s2, "lora t_o gemm"));
    prof_mark(h, s2, T_MISC);
    HIP_TRY(launch_scale_split(L.t_o, (size_t)I.Ti * LR, lora->scale, L.to_hi, nullptr, s2), "lora t_o split");
    HIP_TRY(launch_scale_split(L.t_o + (size_t)I.Ti * LR, (size_t)I.Tf * LR, lora->scale, S.to, L.to_lo, s2), "lora t_o split ft");
    if (s2 != st) prof_mark(h, s2, -1);
  }
  {
    GemmParams p = gp_init(D.qd, D.qd, D.qd, D.d);
    p.resid_kind = resid_x; p.ldr = D.d;
    gp_group(p, S.o, F.o_lo, S.x1, xb + (size_t)I.Ti * D.d * es, I.Tf, np_ft);
    gp_group(p, F.o_i, nullptr, F.x1_i, x, I.Ti, 1);
    gp_seg(p, W.hi[W_O], W.lo[W_O], D.d, 0);
    TRY(run_gemm(h, 0, 0, p, st, "o gemm"));
  }
  if (lora) {
    HIP_TRY(side_join(h, st), "join side stream");
    GemmParams p2 = gp_init(LR, LR, LR, D.d);
    p2.resid_kind = 1; p2.ldr = D.d;
    gp_group(p2, S.to, L.to_lo, S.x1, S.x1, I.Tf, np_ft);
    gp_group(p2, L.to_hi, nullptr, F.x1_i, F.x1_i, I.Ti, 1);
    gp_seg(p2, L.bo_hi, L.bo_lo, D.d, 0);
    TRY(run_gemm(h, 0, 0, p2, st, "lora o gemm"));
  }
  // 6. RMSNorm (MLP), gate/up projection, SwiGLU, down projection + residual
  prof_mark(h, st, T_RMSNORM);
  HIP_TRY(launch_rmsnorm_fwd(F.x1_i, false, nullptr, w->g_mlp, D.bf, I.Ti, D.d, h->m.rms_eps, F.b_i, nullptr, nullptr, st), "rmsnorm2");
  prof_mark(h, st, T_RMSNORM);
  HIP_TRY(launch_rmsnorm_fwd(S.x1, false, nullptr, w->g_mlp, D.bf, I.Tf, D.d, h->m.rms_eps, S.b, F.b_lo, S.rstd2, st), "rmsnorm2 ft");
  {
    // gate and up projections with SwiGLU in the epilogue: hm = silu(G) * U leaves the kernel as bf16
    // (two terms for the fine-tune rows, whose G and U are kept as bf16 for the backward pass)
    GemmParams p = gp_init(D.d, D.d, D.d, D.F);
    p.swiglu = 1; p.out_bf16 = 1;
    gp_group(p, S.b, F.b_lo, S.hm, nullptr, I.Tf, np_ft);
    if (I.Tf > 0) { p.mg[p.n_mg - 1].c_lo = F.hm_lo; p.mg[p.n_mg - 1].c_gu = S.gu; }
    gp_group(p, F.b_i, nullptr, F.hm_i, nullptr, I.Ti, 1);
    gp_seg(p, W.hi[W_G], W.lo[W_G], D.F, 0);
    gp_seg(p, W.hi[W_U], W.lo[W_U], D.F, D.F);
    TRY(run_gemm(h, 0, 0, p, st, "gate/up gemm"));
  }
  {
    GemmParams p = gp_init(D.F, D.F, D.F, D.d);
    p.resid_kind = 1; p.ldr = D.d;
    gp_group(p, S.hm, F.hm_lo, y + (size_t)I.Ti * D.d, S.x1, I.Tf, np_ft);
    gp_group(p, F.hm_i, nullptr, y, F.x1_i, I.Ti, 1);
    gp_seg(p, W.hi[W_D], W.lo[W_D], D.d, 0);
    TRY(run_gemm(h, 0, 0, p, st, "down gemm"));
  }
  prof_mark(h, st, -1);
  return MACE_OK;
}

int mace_hybrid_layer_fwd(mace_handle_t h, const mace_layer_w_t *w, const mace_batch_t *batch, mace_kv_cache_t *cache,
                          const void *x, float *y, void *saved, void *workspace, size_t workspace_bytes, void *stream) {
  return layer_fwd_impl(h, w, nullptr, batch, cache, x, y, saved, workspace, workspace_bytes, stream);
}

int mace_hybrid_layer_fwd_lora(mace_handle_t h, const mace_layer_w_t *w, const mace_lora_t *lora, const mace_batch_t *batch,
                               mace_kv_cache_t *cache, const void *x, float *y, void *saved, void *workspace,
                               size_t workspace_bytes, void *stream) {
  if (!lora) return fail(MACE_INVALID_ARG, "lora is null");
  return layer_fwd_impl(h, w, lora, batch, cache, x, y, saved, workspace, workspace_bytes, stream);
}

static int layer_bwd_impl(mace_handle_t h, const mace_layer_w_t *w, const mace_lora_t *lora, const mace_batch_t *batch,
                          const void *x, const float *dy_ft, const void *saved, float *dx_ft,
                          const mace_layer_grads_t *grads, const mace_lora_grads_t *lgrads, int accumulate,
                          void *workspace, size_t workspace_bytes, void *stream) {
  if (!h || !w || !x || !dy_ft || !saved || !dx_ft || (!grads && !lgrads)) return fail(MACE_INVALID_ARG, "mace_hybrid_layer_bwd: null argument");
  if (lora) TRY(check_lora(lora));
  static const mace_layer_grads_t no_grads = {};
  if (!grads) grads = &no_grads;
  if (!w->g_attn || !w->wq || !w->wk || !w->wv || !w->wo || !w->g_mlp || !w->w_gate || !w->w_up || !w->w_down) return fail(MACE_INVALID_ARG, "null weight pointer");
  BatchInfo I;
  TRY(check_batch(batch, I));
  const Dims D(h->m);
  hipStream_t st = (hipStream_t)stream;
  if (I.Tf == 0) return MACE_OK;
  if (!workspace) return fail(MACE_INVALID_ARG, "workspace is null");
  if (((uintptr_t)workspace & 255) || ((uintptr_t)saved & 255)) return fail(MACE_INVALID_ARG, "workspace/saved must be 256-byte aligned");
  {
    Bump m(nullptr);
    WSplit tmp;
    prepare_weights(D, w, m, false, false, st, tmp);
    plan_bwd(D, I.Tf, m);
    if (lora) plan_lora(D, (size_t)I.Tf, true, m);
    if (m.off > workspace_bytes) return fail(MACE_WORKSPACE_TOO_SMALL, "backward workspace too small");
  }
  SideGuard side_guard(h, st);
  Bump wsb(workspace), svb((void *)saved);
  WSplit W;
  TRY(prepare_weights(D, w, wsb, false, true, st, W));
  BwdWs B = plan_bwd(D, I.Tf, wsb);
  LoraWs L;
  if (lora) {
    L = plan_lora(D, (size_t)I.Tf, true, wsb);
    prof_mark(h, st, T_MISC);
    TRY(prepare_lora(D, lora, L, lora->scale, st));     // B matrices carry the adapter scale here
  }
  const Saved S = plan_saved(D, I.Tf, svb);
  const int Tf = I.Tf;
  const size_t es = D.bf ? 2 : 4;
  const int acc = accumulate ? 1 : 0;
  const int n_part = Tf < DG_PARTS ? Tf : DG_PARTS;

  prof_mark(h, st, T_MISC);
  HIP_TRY(launch_split_f32(dy_ft, (size_t)Tf * D.d, B.dy_bf, nullptr, st), "cast dy");
  // MLP: dHm = dY Wd ; SwiGLU backward ; dWd = dY^T Hm with the Hm the forward kept
  {
    // where the product runs on the four-wave kernel its epilogue does the SwiGLU backward (dHm stays in registers)
    GemmParams pf = gp_init(D.d, D.d, D.F, 2ll * D.F);
    pf.out_bf16 = 1; pf.swiglu_bwd = 1;
    gp_group(pf, B.dy_bf, nullptr, B.dgu, nullptr, Tf, 1);
    pf.mg[0].c_gu = (void *)S.gu;
    gp_seg(pf, W.hi[W_D], nullptr, D.F, 0);
    if (gemm_uses_four_wave(0, 1, pf)) {
      TRY(run_gemm(h, 0, 1, pf, st, "dhm gemm + swiglu bwd"));
    } else {
      GemmParams p = gp_init(D.d, D.d, D.F, D.F);
      p.out_bf16 = 1;
      gp_group(p, B.dy_bf, nullptr, B.dhm, nullptr, Tf, 1);
      gp_seg(p, W.hi[W_D], nullptr, D.F, 0);
      TRY(run_gemm(h, 0, 1, p, st, "dhm gemm"));
      prof_mark(h, st, T_SWIGLU);
      HIP_TRY(launch_swiglu_bwd(B.dhm, S.gu, Tf, D.F, B.dgu, st), "swiglu bwd");
    }
  }
  if (grads->w_down) {
    GemmParams p = gp_init(Tf, D.d, D.F, D.F);
    p.resid_kind = acc;
    gp_group(p, B.dy_bf, nullptr, grads->w_down, grads->w_down, D.d, 1);
    gp_seg(p, S.hm, nullptr, D.F, 0);
    TRY(run_gemm_side(h, 1, 1, p, st, "dWd gemm"));
  }
  // db = dG Wg + dU Wu ; dWg = dG^T b ; dWu = dU^T b
  {
    // one product over the stacked reduction [dG | dU] x [Wg ; Wu]
    GemmParams p = gp_init(2 * D.F, 2 * D.F, D.d, D.d);
    gp_group(p, B.dgu, nullptr, B.db, nullptr, Tf, 1);
    gp_seg(p, W.hi[W_G], nullptr, D.d, 0);
    p.n_kseg = 2;
    p.kseg_b[0] = W.hi[W_G]; p.kseg_b[1] = W.hi[W_U];
    p.kseg_start[0] = 0; p.kseg_start[1] = D.F; p.kseg_start[2] = 2 * D.F;
    TRY(run_gemm(h, 0, 1, p, st, "db gemm"));
  }
  if (grads->w_gate || grads->w_up) {
    GemmParams p = gp_init(Tf, 2 * D.F, D.d, D.d);
    p.resid_kind = acc;
    if (grads->w_gate) gp_group(p, B.dgu, nullptr, grads->w_gate, grads->w_gate, D.F, 1);
    if (grads->w_up) gp_group(p, B.dgu + D.F, nullptr, grads->w_up, grads->w_up, D.F, 1);
    gp_seg(p, S.b, nullptr, D.d, 0);
    TRY(run_gemm_side(h, 1, 1, p, st, "dWg/dWu gemm"));
  }
  // RMSNorm (MLP) backward: dx1 = dy + ...
  prof_mark(h, st, T_RMSNORM);
  HIP_TRY(launch_rmsnorm_bwd(B.db, S.x1, false, nullptr, w->g_mlp, D.bf, S.rstd2, dy_ft, Tf, D.d, B.dx1, B.dx1_bf, B.dg_part, n_part, st), "rmsnorm2 bwd");
  if (grads->g_mlp) { prof_mark(h, st, T_MISC); HIP_TRY(launch_colsum(B.dg_part, n_part, D.d, B.dg_part + (size_t)DG_PARTS * D.d, grads->g_mlp, acc, st), "dg2");
  }
  // attention output projection.  Adapter variant: dt = dx1 (s B_o) is a skinny product that runs
  // beside the main one; then dattn += dt A_o ; dB_o = dx1^T (s t) with the saved s t ; dA_o = dt^T o.
  if (lora) {
    hipStream_t s2 = side_fork(h, st);
    GemmParams p = gp_init(D.d, D.d, LR, LR);
    p.out_bf16 = 1;
    gp_group(p, B.dx1_bf, nullptr, L.dto, nullptr, Tf, 1);
    gp_seg(p, L.bo_hi, nullptr, LR, 0);
    TRY(run_gemm(h, 0, 1, p, s2, "lora dt_o gemm"));
    if (s2 != st) prof_mark(h, s2, -1);
  }
  {
    GemmParams p = gp_init(D.d, D.d, D.qd, D.qd);
    p.out_bf16 = 1;
    gp_group(p, B.dx1_bf, nullptr, B.dattn, nullptr, Tf, 1);
    gp_seg(p, W.hi[W_O], nullptr, D.qd, 0);
    TRY(run_gemm(h, 0, 1, p, st, "dattn gemm"));
  }
  if (grads->wo) {
    GemmParams p = gp_init(Tf, D.d, D.qd, D.qd);
    p.resid_kind = acc;
    gp_group(p, B.dx1_bf, nullptr, grads->wo, grads->wo, D.d, 1);
    gp_seg(p, S.o, nullptr, D.qd, 0);
    TRY(run_gemm_side(h, 1, 1, p, st, "dWo gemm"));
  }
  if (lora) {
    HIP_TRY(side_join(h, st), "join side stream");
    {
      GemmParams p = gp_init(LR, LR, D.qd, D.qd);
      p.out_bf16 = 1; p.resid_kind = 2;
      gp_group(p, L.dto, nullptr, B.dattn, B.dattn, Tf, 1);
      gp_seg(p, L.ao_hi, nullptr, D.qd, 0);
      TRY(run_gemm(h, 0, 1, p, st, "lora dattn gemm"));
    }
    if (lgrads->b_o) {
      hipStream_t s2 = side_fork(h, st);
      GemmParams p = gp_init(Tf, D.d, LR, LR);
      gp_group(p, B.dx1_bf, nullptr, L.dbo, nullptr, D.d, 1);
      gp_seg(p, S.to, nullptr, LR, 0);
      TRY(run_gemm(h, 1, 1, p, s2, "lora dB_o gemm"));
      prof_mark(h, s2, T_MISC);
      HIP_TRY(launch_extract(L.dbo, LR, 0, 0, D.d, lora->rank, 1.0f, lgrads->b_o, acc, s2), "lora dB_o");
      if (s2 != st) prof_mark(h, s2, -1);
    }
    if (lgrads->a_o) {
      hipStream_t s2 = side_fork(h, st);
      GemmParams p = gp_init(Tf, LR, D.qd, D.qd);
      gp_group(p, L.dto, nullptr, L.dao, nullptr, LR, 1);
      gp_seg(p, S.o, nullptr, D.qd, 0);
      TRY(run_gemm(h, 1, 1, p, s2, "lora dA_o gemm"));
      prof_mark(h, s2, T_MISC);
      HIP_TRY(launch_extract(L.dao, D.qd, 0, 0, lora->rank, D.qd, 1.0f, lgrads->a_o, acc, s2), "lora dA_o");
      if (s2 != st) prof_mark(h, s2, -1);
    }
  }
  // attention backward; its epilogues rotate dq and dk back (RoPE backward) and write the bf16 operand of the
  // projection backward directly
  prof_mark(h, st, T_ROPE);
  HIP_TRY(launch_rope_table(batch->positions + I.Ti, h->inv_freq, Tf, D.hd, B.cs, st), "rope table");
  prof_mark(h, st, T_ATTN_BWD, 10.0 * D.hd * D.Hq * I.pairs_ft);
  HIP_TRY(launch_attn_bwd(S.q, S.k, S.v, S.o, B.dattn, S.lse, batch->seg_offsets + batch->n_prefill + batch->n_decode, I.Ti, batch->n_ft_seq, I.max_ft, Tf,
                          D.Hq, D.Hkv, D.hd, B.dvec, B.cs, B.dqkv, st, batch->ft_excl_lo, batch->ft_excl_hi), "attention bwd");
  // da = dq Wq + dk Wk + dv Wv ; dWq, dWk, dWv
  {
    const bf16_t *as[3] = {B.dqkv, B.dqkv + D.qd, B.dqkv + D.qd + D.kd};
    const int ks[3] = {D.qd, D.kd, D.kd};
    const int wi[3] = {W_Q, W_K, W_V};
    if (lora) {
      // q/k/v adapters at once through the stacked A and the block-diagonal (scaled) B: dt beside the main product
      hipStream_t s2 = side_fork(h, st);
      GemmParams p = gp_init(D.nqkv, D.nqkv, 3 * LR, 3 * LR);
      p.out_bf16 = 1;
      gp_group(p, B.dqkv, nullptr, L.dtq, nullptr, Tf, 1);
      gp_seg(p, L.bblk_hi, nullptr, 3 * LR, 0);
      TRY(run_gemm(h, 0, 1, p, s2, "lora dt_qkv gemm"));
      if (s2 != st) prof_mark(h, s2, -1);
    }
    {
      // one product over the stacked reduction [dQ | dK | dV] x [Wq ; Wk ; Wv]
      GemmParams p = gp_init(D.nqkv, D.nqkv, D.d, D.d);
      gp_group(p, B.dqkv, nullptr, B.da, nullptr, Tf, 1);
      gp_seg(p, W.hi[W_Q], nullptr, D.d, 0);
      p.n_kseg = 3;
      for (int i = 0; i < 3; ++i) p.kseg_b[i] = W.hi[wi[i]];
      p.kseg_start[0] = 0; p.kseg_start[1] = ks[0]; p.kseg_start[2] = ks[0] + ks[1]; p.kseg_start[3] = ks[0] + ks[1] + ks[2];
      TRY(run_gemm(h, 0, 1, p, st, "da gemm"));
    }
    if (lora) {
      HIP_TRY(side_join(h, st), "join side stream");
      {
        GemmParams p = gp_init(3 * LR, 3 * LR, D.d, D.d);
        p.resid_kind = 1;
        gp_group(p, L.dtq, nullptr, B.da, B.da, Tf, 1);
        gp_seg(p, L.aqkv_hi, nullptr, D.d, 0);
        TRY(run_gemm(h, 0, 1, p, st, "lora da gemm"));
      }
      if (lgrads->b_q || lgrads->b_k || lgrads->b_v) {
        hipStream_t s2 = side_fork(h, st);
        GemmParams p = gp_init(Tf, D.nqkv, 3 * LR, 3 * LR);
        gp_group(p, B.dqkv, nullptr, L.dbblk, nullptr, D.nqkv, 1);
        gp_seg(p, S.tq, nullptr, 3 * LR, 0);
        TRY(run_gemm(h, 1, 1, p, s2, "lora dB_qkv gemm"));
        float *dst[3] = {lgrads->b_q, lgrads->b_k, lgrads->b_v};
        const int r0[3] = {0, D.qd, D.qd + D.kd}, nr[3] = {D.qd, D.kd, D.kd};
        for (int i = 0; i < 3; ++i)
          if (dst[i]) {
            prof_mark(h, s2, T_MISC);
            HIP_TRY(launch_extract(L.dbblk, 3 * LR, r0[i], i * LR, nr[i], lora->rank, 1.0f, dst[i], acc, s2), "lora dB_qkv");
          }
        if (s2 != st) prof_mark(h, s2, -1);
      }
      if (lgrads->a_q || lgrads->a_k || lgrads->a_v) {
        hipStream_t s2 = side_fork(h, st);
        GemmParams p = gp_init(Tf, 3 * LR, D.d, D.d);
        gp_group(p, L.dtq, nullptr, L.daqkv, nullptr, 3 * LR, 1);
        gp_seg(p, S.a, nullptr, D.d, 0);
        TRY(run_gemm(h, 1, 1, p, s2, "lora dA_qkv gemm"));
        float *dst[3] = {lgrads->a_q, lgrads->a_k, lgrads->a_v};
        for (int i = 0; i < 3; ++i)
          if (dst[i]) {
            prof_mark(h, s2, T_MISC);
            HIP_TRY(launch_extract(L.daqkv, D.d, i * LR, 0, lora->rank, D.d, 1.0f, dst[i], acc, s2), "lora dA_qkv");
          }
        if (s2 != st) prof_mark(h, s2, -1);
      }
    }
    if (grads->wq || grads->wk || grads->wv) {
      GemmParams p = gp_init(Tf, D.nqkv, D.d, D.d);
      p.resid_kind = acc;
      if (grads->wq) gp_group(p, as[0], nullptr, grads->wq, grads->wq, D.qd, 1);
      if (grads->wk) gp_group(p, as[1], nullptr, grads->wk, grads->wk, D.kd, 1);
      if (grads->wv) gp_group(p, as[2], nullptr, grads->wv, grads->wv, D.kd, 1);
      gp_seg(p, S.a, nullptr, D.d, 0);
      TRY(run_gemm_side(h, 1, 1, p, st, "dWqkv gemm"));
    }
  }
  // RMSNorm (attention) backward: dx = dx1 + ...
  prof_mark(h, st, T_RMSNORM);
  HIP_TRY(launch_rmsnorm_bwd(B.da, (const char *)x + (size_t)I.Ti * D.d * es, D.bf, nullptr, w->g_attn, D.bf, S.rstd1, B.dx1, Tf, D.d, dx_ft, nullptr, B.dg_part, n_part, st), "rmsnorm1 bwd");
  if (grads->g_attn) { prof_mark(h, st, T_MISC); HIP_TRY(launch_colsum(B.dg_part, n_part, D.d, B.dg_part + (size_t)DG_PARTS * D.d, grads->g_attn, acc, st), "dg1");
  }
  prof_mark(h, st, -1);
  HIP_TRY(side_join(h, st), "join side stream");
  return MACE_OK;
}

int mace_hybrid_layer_bwd(mace_handle_t h, const mace_layer_w_t *w, const mace_batch_t *batch, const void *x,
                          const float *dy_ft, const void *saved, float *dx_ft, const mace_layer_grads_t *grads,
                          int accumulate, void *workspace, size_t workspace_bytes, void *stream) {
  if (!grads) return fail(MACE_INVALID_ARG, "mace_hybrid_layer_bwd: null argument");
  return layer_bwd_impl(h, w, nullptr, batch, x, dy_ft, saved, dx_ft, grads, nullptr, accumulate, workspace, workspace_bytes, stream);
}

int mace_hybrid_layer_bwd_lora(mace_handle_t h, const mace_layer_w_t *w, const mace_lora_t *lora, const mace_batch_t *batch,
                               const void *x, const float *dy_ft, const void *saved, float *dx_ft,
                               const mace_lora_grads_t *grads, int accumulate, void *workspace, size_t workspace_bytes,
                               void *stream) {
  if (!lora || !grads) return fail(MACE_INVALID_ARG, "mace_hybrid_layer_bwd_lora: null argument");
  return layer_bwd_impl(h, w, lora, batch, x, dy_ft, saved, dx_ft, nullptr, grads, accumulate, workspace, workspace_bytes, stream);
}

// chosen_lens / chosen_lens_host non-null selects the shared-prompt layout: offsets and prompt
// lengths are then per PAIR (prompt | chosen | rejected stored once).
static int dpo_impl(mace_handle_t h, const float *h_ft, const void *g_final, const void *w_lm,
                    const int32_t *token_ids, const int32_t *ft_seq_offsets, const int32_t *ft_seq_offsets_host,
                    const int32_t *prompt_lens, const int32_t *prompt_lens_host, const int32_t *chosen_lens,
                    const int32_t *chosen_lens_host, int32_t n_pairs,
                    const float *ref_logp, float beta, float *logp_out, float *loss_per_pair, float *loss_mean,
                    float *clpd_out, int32_t *win_out, float *dh_ft, float *dw_lm, float *dg_final, int accumulate,
                    void *workspace, size_t workspace_bytes, void *stream) {
  if (!h || !h_ft || !g_final || !w_lm || !token_ids || !ft_seq_offsets || !ft_seq_offsets_host || !prompt_lens || !prompt_lens_host ||
      !ref_logp || !logp_out || !loss_per_pair || !loss_mean)
    return fail(MACE_INVALID_ARG, "mace_dpo_logprob_loss: null argument");
  if (n_pairs <= 0 || n_pairs > 32767) return fail(MACE_INVALID_ARG, "n_pairs must be in 1..32767");
  if (!std::isfinite(beta)) return fail(MACE_INVALID_ARG, "beta");
  const bool shared = chosen_lens_host != nullptr;
  if (shared && !chosen_lens) return fail(MACE_INVALID_ARG, "chosen_lens device pointer is null");
  const Dims D(h->m);
  const int n_seq = 2 * n_pairs;
  const int n_stored = shared ? n_pairs : n_seq;       // stored row ranges
  if (ft_seq_offsets_host[0] != 0) return fail(MACE_INVALID_ARG, "ft_seq_offsets must start at 0");
  long long R = 0;
  for (int s = 0; s < n_stored; ++s) {
    const int L = ft_seq_offsets_host[s + 1] - ft_seq_offsets_host[s], P = prompt_lens_host[s];
    if (L < 1 || P < 1 || P > L) return fail(MACE_INVALID_ARG, "need 1 <= prompt_len <= sequence length");
    if (shared && (chosen_lens_host[s] < 1 || L - P - chosen_lens_host[s] < 1)) return fail(MACE_INVALID_ARG, "both responses of a pair need at least one token");
    R += L - P;
  }
  if (R > INT32_MAX / 2) return fail(MACE_INVALID_ARG, "too many loss rows");
  const int Tf = ft_seq_offsets_host[n_stored];
  if (!workspace || ((uintptr_t)workspace & 255)) return fail(MACE_INVALID_ARG, "workspace must be non-null and 256-byte aligned");
  {
    Bump m(nullptr);
    plan_dpo(D, (size_t)R, n_seq, m);
    if (m.off > workspace_bytes) return fail(MACE_WORKSPACE_TOO_SMALL, "DPO workspace too small");
  }
  hipStream_t st = (hipStream_t)stream;
  SideGuard side_guard(h, st);
  Bump wsb(workspace);
  DpoWs P = plan_dpo(D, (size_t)R, n_seq, wsb);
  const bf16_t *e_hi = (const bf16_t *)w_lm, *e_lo = nullptr;
  if (!D.bf) {
    prof_mark(h, st, T_MISC);
    HIP_TRY(launch_split_f32((const float *)w_lm, (size_t)D.V * D.d, P.e_hi, P.e_lo, st), "split head");
    e_hi = P.e_hi; e_lo = P.e_lo;
  }
  const int Ri = (int)R;
  const bool want_grad = dh_ft || dw_lm || dg_final;
  const int acc = accumulate ? 1 : 0;
  // Head precision.  fp32 weights: three-product form.  bf16 weights, MACE_OPT_HEAD_TWO_PASS or no gradient
  // wanted: two passes over the vocabulary (two-term activations).  bf16 weights with gradients (the default
  // of a training step): ONE pass with n_hi, and the first-order term of the dropped n_lo is added to every
  // row's log-probability from u = dl E, the product the backward pass forms anyway (logp_correct_kernel).
  const bool one_pass = D.bf && !h->head_two_pass && want_grad;
  // without dh_ft the two-sequence layout writes the row gradients over the logits buffer (the shared layout
  // writes them densely over dn and needs no such room)
  if (dg_final && !dh_ft && !shared && (size_t)Tf * D.d > (size_t)Ri * D.V) return fail(MACE_INVALID_ARG, "dg_final without dh_ft needs T_f*d <= R*V");
  const bool need_u = Ri > 0 && want_grad && (dh_ft || dg_final || one_pass);
  if (Ri > 0) {
    prof_mark(h, st, T_MISC);
    if (shared)
      HIP_TRY(launch_loss_rows_shared(ft_seq_offsets, prompt_lens, chosen_lens, token_ids, n_pairs, P.row_idx, P.label, P.seq_id, P.partner,
                                      P.vseq_off, P.vprompt, st), "loss rows (shared prompt)");
    else
      HIP_TRY(launch_loss_rows(ft_seq_offsets, prompt_lens, token_ids, n_seq, P.row_idx, P.label, P.seq_id, st), "loss rows");
    prof_mark(h, st, T_RMSNORM);
    HIP_TRY(launch_rmsnorm_fwd(h_ft, false, P.row_idx, g_final, D.bf, Ri, D.d, h->m.rms_eps, P.n_hi, P.n_lo, P.rstd, st), "final rmsnorm");
    GemmParams p = gp_init(D.d, D.d, D.d, D.V);
    gp_group(p, P.n_hi, P.n_lo, P.logits, nullptr, Ri, one_pass ? 1 : (D.bf ? 2 : 3));
    gp_seg(p, e_hi, e_lo, D.V, 0);
    TRY(run_gemm(h, 0, 0, p, st, "lm head gemm"));
    // log-soft-max and, for the backward, dl = onehot - softmax (without the sequence factor) in one pass over the logits
    prof_mark(h, st, T_LOGSOFTMAX, 0.0, (double)Ri * D.V * (want_grad ? 6.0 : 4.0));
    HIP_TRY(launch_logsoftmax_dl(P.logits, Ri, D.V, P.label, P.logp_t, P.lse, want_grad ? P.dl : nullptr, st), "log-softmax");
    if (need_u) {
      // u = dl E: small output, reduction over the whole vocabulary: slice k so that every CU has work
      const int ks = gemm_suggest_k_splits(Ri, D.d, D.V);
      GemmParams q = gp_init(D.V, D.V, D.d, D.d);
      gp_group(q, P.dl, nullptr, ks > 1 ? P.dn_part : P.dn, nullptr, Ri, 1);
      gp_seg(q, e_hi, nullptr, D.d, 0);
      if (ks > 1) { q.k_splits = ks; q.c_split_stride = (long long)Ri * D.d; }
      TRY(run_gemm(h, 0, 1, q, st, "dn gemm"));
      if (ks > 1) { prof_mark(h, st, T_MISC); HIP_TRY(launch_sum_partials(P.dn_part, ks, (size_t)Ri * D.d, P.dn, st), "dn partial sums"); }
      if (one_pass) { prof_mark(h, st, T_MISC); HIP_TRY(launch_logp_correct(P.n_lo, P.dn, Ri, D.d, P.logp_t, st), "log-probability correction"); }
    }
  }
  prof_mark(h, st, T_MISC);
  HIP_TRY(launch_dpo_pairs(P.logp_t, shared ? P.vseq_off : ft_seq_offsets, shared ? P.vprompt : prompt_lens, n_seq, ref_logp, beta, logp_out, loss_per_pair, loss_mean, clpd_out, win_out, P.dlogp, st), "dpo pairs");
  if (!want_grad) { prof_mark(h, st, -1); return MACE_OK; }
  if (dh_ft) { prof_mark(h, st, T_MISC); HIP_TRY(launch_fill_f32(dh_ft, (size_t)Tf * D.d, 0.f, st), "zero dh");
  }
  if (Ri == 0) {
    if (!acc) {
      if (dw_lm) { prof_mark(h, st, T_MISC); HIP_TRY(launch_fill_f32(dw_lm, (size_t)D.V * D.d, 0.f, st), "zero dE");
  }
      if (dg_final) { prof_mark(h, st, T_MISC); HIP_TRY(launch_fill_f32(dg_final, (size_t)D.d, 0.f, st), "zero dg");
  }
    }
    prof_mark(h, st, -1);
    return MACE_OK;
  }
  // the sequence factor c = dL/dlog p, known now: dn = c u; dE = dl^T (c n_hi), the scaled rows take the place of n_lo
  bf16_t *n_c = dw_lm ? P.n_lo : nullptr;
  prof_mark(h, st, T_MISC);
  HIP_TRY(launch_scale_rows(dh_ft || dg_final ? P.dn : nullptr, P.n_hi, n_c, P.seq_id, P.dlogp, Ri, D.d, st), "sequence factors");
  if (dw_lm) {
    GemmParams p = gp_init(Ri, D.V, D.d, D.d);
    p.resid_kind = acc;
    gp_group(p, P.dl, nullptr, dw_lm, dw_lm, D.V, 1);
    gp_seg(p, n_c, nullptr, D.d, 0);
    TRY(run_gemm_side(h, 1, 1, p, st, "dE gemm"));
  }
  if (dh_ft || dg_final) {
    const int n_part = Ri < DG_PARTS ? Ri : DG_PARTS;
    // without dh_ft the row gradients still have to land somewhere: reuse the logits buffer
    float *dx_dst = dh_ft ? dh_ft : P.logits;
    prof_mark(h, st, T_RMSNORM);
    if (shared) {
      // two loss rows of a pair (the first token of either response) land on the same stored row: norm backward
      // in place on the dense rows, then a scatter that adds the two
      HIP_TRY(launch_rmsnorm_bwd(P.dn, h_ft, false, P.row_idx, g_final, D.bf, P.rstd, nullptr, Ri, D.d, P.dn, nullptr, P.dg_part, n_part, st, 1), "final rmsnorm bwd");
      if (dh_ft) { prof_mark(h, st, T_MISC); HIP_TRY(launch_scatter_rows(P.dn, P.row_idx, P.partner, Ri, D.d, dh_ft, st), "scatter dh");
      }
    } else
    HIP_TRY(launch_rmsnorm_bwd(P.dn, h_ft, false, P.row_idx, g_final, D.bf, P.rstd, nullptr, Ri, D.d, dx_dst, nullptr, P.dg_part, n_part, st), "final rmsnorm bwd");
    if (dg_final) { prof_mark(h, st, T_MISC); HIP_TRY(launch_colsum(P.dg_part, n_part, D.d, P.dg_part + (size_t)DG_PARTS * D.d, dg_final, acc, st), "dg_final");
    }
  }
  prof_mark(h, st, -1);
  HIP_TRY(side_join(h, st), "join side stream");
  return MACE_OK;
}

int mace_dpo_logprob_loss(mace_handle_t h, const float *h_ft, const void *g_final, const void *w_lm,
                          const int32_t *token_ids, const int32_t *ft_seq_offsets, const int32_t *ft_seq_offsets_host,
                          const int32_t *prompt_lens, const int32_t *prompt_lens_host, int32_t n_pairs,
                          const float *ref_logp, float beta, float *logp_out, float *loss_per_pair, float *loss_mean,
                          float *clpd_out, int32_t *win_out, float *dh_ft, float *dw_lm, float *dg_final, int accumulate,
                          void *workspace, size_t workspace_bytes, void *stream) {
  return dpo_impl(h, h_ft, g_final, w_lm, token_ids, ft_seq_offsets, ft_seq_offsets_host, prompt_lens, prompt_lens_host, nullptr, nullptr,
                  n_pairs, ref_logp, beta, logp_out, loss_per_pair, loss_mean, clpd_out, win_out, dh_ft, dw_lm, dg_final, accumulate,
                  workspace, workspace_bytes, stream);
}

int mace_dpo_logprob_loss_shared(mace_handle_t h, const float *h_ft, const void *g_final, const void *w_lm,
                                 const int32_t *token_ids, const int32_t *pair_offsets, const int32_t *pair_offsets_host,
                                 const int32_t *prompt_lens, const int32_t *prompt_lens_host, const int32_t *chosen_lens,
                                 const int32_t *chosen_lens_host, int32_t n_pairs, const float *ref_logp, float beta,
                                 float *logp_out, float *loss_per_pair, float *loss_mean, float *clpd_out, int32_t *win_out,
                                 float *dh_ft, float *dw_lm, float *dg_final, int accumulate, void *workspace,
                                 size_t workspace_bytes, void *stream) {
  if (!chosen_lens || !chosen_lens_host) return fail(MACE_INVALID_ARG, "mace_dpo_logprob_loss_shared: null argument");
  return dpo_impl(h, h_ft, g_final, w_lm, token_ids, pair_offsets, pair_offsets_host, prompt_lens, prompt_lens_host, chosen_lens,
                  chosen_lens_host, n_pairs, ref_logp, beta, logp_out, loss_per_pair, loss_mean, clpd_out, win_out, dh_ft, dw_lm, dg_final,
                  accumulate, workspace, workspace_bytes, stream);
}

}  // extern "C"
