"""Seeded synthetic workloads for one hybrid iteration (prefill + decode + DPO rows).

This module only draws numbers and lays out index arrays.  It holds none of the
method's arithmetic (no norm, attention, soft-max or loss) and is shared by the
tests of the CPU oracle and of the HIP path so that both consume the very same
inputs.  It depends on numpy only.

The five workloads stand in for the preference data (HH-RLHF, SHP) and the
7B-class / edge models the paper serves (Section 6.1): shapes, length mixes and
value distributions are those of the benchmark configurations, token ids are
uniform over the vocabulary and no dataset text is used.

Random numbers come from a counter-based generator: value i of stream s under
seed S is a function of (S, s, i) alone (splitmix64 finaliser, then Box-Muller
for normals), so any slice can be regenerated without generating the rest.
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional

import numpy as np

_U64 = np.uint64
_GOLD = _U64(0x9E3779B97F4A7C15)

# Fixed stream numbering (order documented with the workload recipe).
STREAMS = {
    "E": 0, "g1": 1, "wq": 2, "wk": 3, "wv": 4, "wo": 5, "g2": 6, "wg": 7, "wu": 8,
    "wd": 9, "gf": 10, "prefill_len": 11, "decode_ctx": 12, "resp_len": 13,
    "token_ids": 14, "cache_k": 15, "cache_v": 16, "ref_logp": 17, "block_perm": 18,
    "dy": 19,
    "lora_a_q": 20, "lora_b_q": 21, "lora_a_k": 22, "lora_b_k": 23, "lora_a_v": 24, "lora_b_v": 25,
    "lora_a_o": 26, "lora_b_o": 27, "prefix_k": 28, "prefix_v": 29,
}


def _mix(z: np.ndarray) -> np.ndarray:
    """splitmix64 output function on a uint64 array (wrap-around arithmetic)."""
    z = (z ^ (z >> _U64(30))) * _U64(0xBF58476D1CE4E5B9)
    z = (z ^ (z >> _U64(27))) * _U64(0x94D049BB133111EB)
    return z ^ (z >> _U64(31))


def raw_u64(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """`count` 64-bit words of stream `stream`, counters start..start+count-1."""
    with np.errstate(over="ignore"):
        base = _mix(_U64(seed) * _GOLD + _U64(stream) * _U64(0xD1B54A32D192ED03) + _U64(0x632BE59BD9B4E019))
        idx = np.arange(start, start + count, dtype=np.uint64)
        return _mix(base + (idx + _U64(1)) * _GOLD)


def uniform01(seed: int, stream: int, start: int, count: int) -> np.ndarray:
    """Uniform doubles in (0, 1): top 53 bits, offset by half an ulp."""
    return ((raw_u64(seed, stream, start, count) >> _U64(11)).astype(np.float64) + 0.5) * (1.0 / 9007199254740992.0)


def normal(seed: int, stream: int, start: int, count: int, chunk: int = 1 << 22) -> np.ndarray:
    """Standard normals.  Value i uses counters 2i and 2i+1 (Box-Muller, cosine branch)."""
    out = np.empty(count, dtype=np.float64)
    for c0 in range(0, count, chunk):
        n = min(chunk, count - c0)
        u = uniform01(seed, stream, 2 * (start + c0), 2 * n)
        out[c0:c0 + n] = np.sqrt(-2.0 * np.log(u[0::2])) * np.cos(2.0 * np.pi * u[1::2])
    return out


def randint(seed: int, stream: int, start: int, count: int, lo: int, hi: int) -> np.ndarray:
    """Uniform integers in [lo, hi], both ends included."""
    span = _U64(hi - lo + 1)
    return (raw_u64(seed, stream, start, count) % span).astype(np.int64) + lo


def permutation(seed: int, stream: int, n: int) -> np.ndarray:
    """A permutation of 0..n-1: argsort of n distinct-with-probability-1 words."""
    return np.argsort(raw_u64(seed, stream, 0, n), kind="stable").astype(np.int64)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bf16 value (ties to even); result held in float32."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    b = f.view(np.uint32)
    r = ((b + np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1))) & np.uint32(0xFFFF0000))
    return r.view(np.float32).reshape(f.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    f = np.ascontiguousarray(x, dtype=np.float32)
    b = f.view(np.uint32)
    assert not np.any(b & np.uint32(0xFFFF)), "value is not bf16-representable"
    return (b >> np.uint32(16)).astype(np.uint16).reshape(f.shape)


@dataclasses.dataclass
class ModelDims:
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    vocab: int
    rms_eps: float = 1e-6
    rope_theta: float = 1e4
    io_bf16: bool = True   # False: fp32 buffers at the boundary (tiny configuration)


@dataclasses.dataclass
class ConfigSpec:
    name: str
    seed: int
    dims: ModelDims
    prefill_lens: Optional[List[int]]      # fixed lengths, or None when drawn
    prefill_draw: Optional[tuple]          # (count, lo, hi)
    decode_ctx: Optional[List[int]]
    decode_draw: Optional[tuple]
    n_pairs: int
    prompt_len: int
    resp_fixed: Optional[int]
    resp_draw: Optional[tuple]             # (lo, hi)
    beta: float = 0.1
    ref_mode: str = "len"                  # "fixed64": N(-64, 4);  "len": N(-2 len, 0.5 sqrt(len))
    block_size: int = 16
    prefill_prefix: Optional[List[int]] = None   # tokens of each prefill request that are already cached (prefix sharing)


_D7B = dict(d_model=4096, n_q_heads=32, n_kv_heads=32, head_dim=128, d_ff=11008, vocab=32000)

CONFIGS: Dict[str, ConfigSpec] = {
    "tiny": ConfigSpec("tiny", 0, ModelDims(256, 4, 4, 64, 704, 2048, io_bf16=False),
                       [48, 64], None, [32, 64, 96, 128], None, 1, 32, 32, None, ref_mode="fixed64"),
    "edge": ConfigSpec("edge", 1, ModelDims(2048, 32, 8, 64, 5632, 32000),
                       None, (8, 128, 512), None, (32, 256, 2048), 4, 256, None, (64, 256)),
    "7b": ConfigSpec("7b", 2, ModelDims(**_D7B), [1024] * 4, None, None, (64, 1024, 4096), 8, 512, 256, None),
    "7b_decode": ConfigSpec("7b_decode", 3, ModelDims(**_D7B), [], None, None, (256, 2048, 8192), 2, 256, 128, None),
    "7b_ft": ConfigSpec("7b_ft", 4, ModelDims(**_D7B), [512] * 2, None, None, (16, 512, 2048), 32, 512, 512, None),
}
CONFIG_ORDER = ["tiny", "edge", "7b", "7b_decode", "7b_ft"]


@dataclasses.dataclass
class Batch:
    """Index side of one iteration.  Rows are ordered prefill | decode | fine-tune."""
    prefill_lens: np.ndarray        # [n_prefill]
    decode_ctx: np.ndarray          # [n_decode] tokens already cached, the new token has this position
    ft_lens: np.ndarray             # [n_ft_seq] sequence 2i = prompt+chosen, 2i+1 = prompt+rejected
    ft_prompt_lens: np.ndarray      # [n_ft_seq]
    seg_offsets: np.ndarray         # [n_prefill+n_decode+n_ft_seq+1] int32 row offsets
    positions: np.ndarray           # [T] int32
    token_ids: np.ndarray           # [T] int32
    block_size: int
    num_blocks: int
    prefill_block_tables: List[np.ndarray]   # per prefill request, int32 block ids
    decode_block_tables: np.ndarray          # [n_decode, max_blocks_per_req] int32, -1 padded
    max_blocks_per_req: int
    prefill_prefix_lens: Optional[np.ndarray] = None   # [n_prefill] cached prefix tokens, None = no prefix anywhere
    ft_chosen_lens: Optional[np.ndarray] = None        # shared-prompt layout: one stored sequence per pair,
                                                       # prompt | chosen response | rejected response; [n_pairs] chosen lengths

    @property
    def n_prefill(self): return len(self.prefill_lens)
    @property
    def n_decode(self): return len(self.decode_ctx)
    @property
    def n_ft_seq(self): return len(self.ft_lens)
    @property
    def t_prefill(self): return int(self.prefill_lens.sum())
    @property
    def t_decode(self): return self.n_decode
    @property
    def t_ft(self): return int(self.ft_lens.sum())
    @property
    def n_tokens(self): return self.t_prefill + self.t_decode + self.t_ft
    @property
    def n_loss_rows(self): return int((self.ft_lens - self.ft_prompt_lens).sum())


@dataclasses.dataclass
class Workload:
    spec: ConfigSpec
    dims: ModelDims
    weights: Dict[str, np.ndarray]   # float32 (bf16-representable when dims.io_bf16)
    batch: Batch
    x: np.ndarray                    # [T, d] float32: embedding rows of token_ids (tied head)
    ctx_k: Optional[List[np.ndarray]]   # per decode request [ctx, Hkv, hd] float32 (post-RoPE keys)
    ctx_v: Optional[List[np.ndarray]]
    ref_logp: np.ndarray             # [n_ft_seq] float32
    beta: float
    pre_k: Optional[List[np.ndarray]] = None   # per prefill request [prefix, Hkv, hd] float32: its cached prefix
    pre_v: Optional[List[np.ndarray]] = None


def _maybe_bf16(a: np.ndarray, io_bf16: bool) -> np.ndarray:
    a = a.astype(np.float32)
    return round_to_bf16(a) if io_bf16 else a


def make_weights(spec: ConfigSpec) -> Dict[str, np.ndarray]:
    """Matrices N(0, 0.02) stored [out, in]; gains 1 + N(0, 0.02); E is the tied embedding/head."""
    m, s = spec.dims, spec.seed
    qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    shapes = {"E": (m.vocab, m.d_model), "wq": (qd, m.d_model), "wk": (kvd, m.d_model), "wv": (kvd, m.d_model),
              "wo": (m.d_model, qd), "wg": (m.d_ff, m.d_model), "wu": (m.d_ff, m.d_model), "wd": (m.d_model, m.d_ff)}
    w = {}
    for name, shp in shapes.items():
        w[name] = _maybe_bf16(0.02 * normal(s, STREAMS[name], 0, shp[0] * shp[1]).reshape(shp), m.io_bf16)
    for name in ("g1", "g2", "gf"):
        w[name] = _maybe_bf16(1.0 + 0.02 * normal(s, STREAMS[name], 0, m.d_model), m.io_bf16)
    return w


def make_lora(spec: ConfigSpec, rank: int = 16, scale: float = 2.0) -> Dict[str, object]:
    """Low-rank adapters on the four attention projections: for projection p with weight
    [out, in], a_p [rank, in] and b_p [out, rank], both N(0, 0.02) (b is non-zero on purpose so
    that every term of the adapter arithmetic is exercised), stored in the io dtype."""
    m, s = spec.dims, spec.seed
    qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    io = {"q": (qd, m.d_model), "k": (kvd, m.d_model), "v": (kvd, m.d_model), "o": (m.d_model, qd)}
    lora: Dict[str, object] = {"rank": int(rank), "scale": float(scale)}
    for pn, (n_out, n_in) in io.items():
        lora["a_" + pn] = _maybe_bf16(0.02 * normal(s, STREAMS["lora_a_" + pn], 0, rank * n_in).reshape(rank, n_in), m.io_bf16)
        lora["b_" + pn] = _maybe_bf16(0.02 * normal(s, STREAMS["lora_b_" + pn], 0, n_out * rank).reshape(n_out, rank), m.io_bf16)
    return lora


def make_batch(spec: ConfigSpec, n_prefill=None, n_decode=None, n_pairs=None) -> Batch:
    """Lengths, positions, token ids and block tables.  The optional counts keep only the
    first requests of each class (request-subsampled batch with per-request shapes unchanged)."""
    s, m = spec.seed, spec.dims
    if spec.prefill_lens is not None:
        pl = np.array(spec.prefill_lens, dtype=np.int64)
    else:
        c, lo, hi = spec.prefill_draw
        pl = randint(s, STREAMS["prefill_len"], 0, c, lo, hi)
    if spec.decode_ctx is not None:
        dc = np.array(spec.decode_ctx, dtype=np.int64)
    else:
        c, lo, hi = spec.decode_draw
        dc = randint(s, STREAMS["decode_ctx"], 0, c, lo, hi)
    npairs = spec.n_pairs
    if spec.resp_fixed is not None:
        rl = np.full(2 * npairs, spec.resp_fixed, dtype=np.int64)
    else:
        lo, hi = spec.resp_draw
        rl = randint(s, STREAMS["resp_len"], 0, 2 * npairs, lo, hi)
    px = np.array(spec.prefill_prefix, dtype=np.int64) if spec.prefill_prefix is not None else None
    if px is not None and len(px) != len(pl):
        raise ValueError("prefill_prefix needs one entry per prefill request")
    if n_prefill is not None:
        px = px[:n_prefill] if px is not None else None
    if n_prefill is not None: pl = pl[:n_prefill]
    if n_decode is not None: dc = dc[:n_decode]
    if n_pairs is not None: rl = rl[:2 * n_pairs]; npairs = n_pairs
    ft_prompt = np.full(2 * npairs, spec.prompt_len, dtype=np.int64)
    ft_lens = ft_prompt + rl

    seg_lens = np.concatenate([pl, np.ones(len(dc), dtype=np.int64), ft_lens])
    seg_offsets = np.concatenate([[0], np.cumsum(seg_lens)]).astype(np.int32)
    T = int(seg_offsets[-1])
    pos = np.empty(T, dtype=np.int32)
    for i, L in enumerate(pl):
        pos[seg_offsets[i]:seg_offsets[i + 1]] = np.arange(L) + (int(px[i]) if px is not None else 0)
    for j, n in enumerate(dc):
        pos[seg_offsets[len(pl) + j]] = n
    for q, L in enumerate(ft_lens):
        o = seg_offsets[len(pl) + len(dc) + q]
        pos[o:o + L] = np.arange(L)

    # Token ids: uniform over the vocabulary; the two sequences of a pair share their prompt.
    tok = randint(s, STREAMS["token_ids"], 0, T, 0, m.vocab - 1).astype(np.int32)
    for i in range(npairs):
        o0 = seg_offsets[len(pl) + len(dc) + 2 * i]
        o1 = seg_offsets[len(pl) + len(dc) + 2 * i + 1]
        tok[o1:o1 + spec.prompt_len] = tok[o0:o0 + spec.prompt_len]

    # Paged cache: each request owns ceil(tokens/B) blocks drawn from one seeded permutation of
    # the pool (a fragmented pool, as after a long run of a server).
    B = spec.block_size
    nb_pre = [int(-(-(L + (int(px[i]) if px is not None else 0)) // B)) for i, L in enumerate(pl)]
    nb_dec = [int(-(-(n + 1) // B)) for n in dc]
    need = sum(nb_pre) + sum(nb_dec)
    num_blocks = need + max(4, need // 8)
    perm = permutation(s, STREAMS["block_perm"], num_blocks)
    cur = 0
    pbt = []
    for nb in nb_pre:
        pbt.append(perm[cur:cur + nb].astype(np.int32)); cur += nb
    mb = max(nb_dec) if nb_dec else 1
    dbt = np.full((len(dc), mb), -1, dtype=np.int32)
    for j, nb in enumerate(nb_dec):
        dbt[j, :nb] = perm[cur:cur + nb]; cur += nb
    return Batch(pl, dc, ft_lens, ft_prompt, seg_offsets, pos, tok, B, num_blocks, pbt, dbt, mb, px)


def make_cached_context(spec: ConfigSpec, batch: Batch):
    """Cached K and V of the decode requests, N(0,1), one contiguous [ctx, Hkv, hd] pair per
    request (each side places them into its paged cache with its own append).  Request j,
    position p, kv head h, element e is value ((off_j + p) * Hkv + h) * hd + e of the stream,
    off_j = sum of the contexts of the requests before j."""
    m = spec.dims
    row = m.n_kv_heads * m.head_dim
    off = 0
    ks, vs = [], []
    for n in batch.decode_ctx:
        n = int(n)
        ks.append(_maybe_bf16(normal(spec.seed, STREAMS["cache_k"], off * row, n * row), m.io_bf16).reshape(n, m.n_kv_heads, m.head_dim))
        vs.append(_maybe_bf16(normal(spec.seed, STREAMS["cache_v"], off * row, n * row), m.io_bf16).reshape(n, m.n_kv_heads, m.head_dim))
        off += n
    return ks, vs


def make_cached_prefix(spec: ConfigSpec, batch: Batch):
    """Cached K and V of the shared prefixes of the prefill requests, N(0,1), laid out like
    make_cached_context (streams prefix_k / prefix_v)."""
    m = spec.dims
    row = m.n_kv_heads * m.head_dim
    off = 0
    ks, vs = [], []
    for n in batch.prefill_prefix_lens:
        n = int(n)
        ks.append(_maybe_bf16(normal(spec.seed, STREAMS["prefix_k"], off * row, n * row), m.io_bf16).reshape(n, m.n_kv_heads, m.head_dim))
        vs.append(_maybe_bf16(normal(spec.seed, STREAMS["prefix_v"], off * row, n * row), m.io_bf16).reshape(n, m.n_kv_heads, m.head_dim))
        off += n
    return ks, vs


def make_ref_logp(spec: ConfigSpec, batch: Batch) -> np.ndarray:
    z = normal(spec.seed, STREAMS["ref_logp"], 0, batch.n_ft_seq)
    if spec.ref_mode == "fixed64":
        r = -64.0 + 4.0 * z
    else:
        ln = (batch.ft_lens - batch.ft_prompt_lens).astype(np.float64)
        r = -2.0 * ln + 0.5 * np.sqrt(ln) * z
    return r.astype(np.float32)


def make_workload(name: str, n_prefill=None, n_decode=None, n_pairs=None, with_cache=True,
                  weights: Optional[Dict[str, np.ndarray]] = None) -> Workload:
    spec = CONFIGS[name]
    w = weights if weights is not None else make_weights(spec)
    b = make_batch(spec, n_prefill, n_decode, n_pairs)
    x = w["E"][b.token_ids]
    ck, cv = make_cached_context(spec, b) if with_cache else (None, None)
    pk, pv = make_cached_prefix(spec, b) if (with_cache and b.prefill_prefix_lens is not None) else (None, None)
    return Workload(spec, spec.dims, w, b, x, ck, cv, make_ref_logp(spec, b), spec.beta, pk, pv)


def to_shared_prompt(wl: Workload) -> Workload:
    """The same workload with every preference pair stored once as prompt | chosen response |
    rejected response (the two sequences of a pair share their prompt tokens, so nothing is lost):
    same tokens, same positions (both responses start at position P), same ref_logp, 2 P + Rc + Rr
    rows per pair become P + Rc + Rr."""
    b = wl.batch
    base = b.n_prefill + b.n_decode
    n_pairs = b.n_ft_seq // 2
    seg = b.seg_offsets
    Ti = int(seg[base])
    rows, pos, lens, chosen, prompts = [], [], [], [], []
    for i in range(n_pairs):
        o0, o1, o2 = int(seg[base + 2 * i]), int(seg[base + 2 * i + 1]), int(seg[base + 2 * i + 2])
        P = int(b.ft_prompt_lens[2 * i])
        assert P == int(b.ft_prompt_lens[2 * i + 1]) and np.array_equal(b.token_ids[o0:o0 + P], b.token_ids[o1:o1 + P])
        rows += list(range(o0, o1)) + list(range(o1 + P, o2))
        Rc, Rr = o1 - o0 - P, o2 - o1 - P
        pos += list(range(P + Rc)) + list(range(P, P + Rr))
        lens.append(P + Rc + Rr); chosen.append(Rc); prompts.append(P)
    rows = np.array(rows, dtype=np.int64)
    keep = np.concatenate([np.arange(Ti), rows])
    ft_lens = np.array(lens, dtype=np.int64)
    seg_new = np.concatenate([seg[:base + 1], Ti + np.cumsum(ft_lens)]).astype(np.int32)
    nb = dataclasses.replace(b, ft_lens=ft_lens, ft_prompt_lens=np.array(prompts, dtype=np.int64), seg_offsets=seg_new,
                             positions=np.concatenate([b.positions[:Ti], np.array(pos, dtype=np.int32)]).astype(np.int32),
                             token_ids=b.token_ids[keep], ft_chosen_lens=np.array(chosen, dtype=np.int64))
    return dataclasses.replace(wl, batch=nb, x=wl.x[keep])


def ft_slice(wl: Workload, p0: int, p1: int) -> Workload:
    """The fine-tune-only batch made of pairs p0 .. p1-1 of `wl` (two-sequence layout): the same rows,
    tokens, positions and reference log-probabilities, no inference rows and an empty cache.  Pure
    index slicing; used to run a part of a large batch on its own."""
    b = wl.batch
    assert b.ft_chosen_lens is None and 0 <= p0 < p1 <= b.n_ft_seq // 2
    base = b.n_prefill + b.n_decode
    seg = b.seg_offsets
    o0, o1 = int(seg[base + 2 * p0]), int(seg[base + 2 * p1])
    nb = Batch(np.zeros(0, np.int64), np.zeros(0, np.int64), b.ft_lens[2 * p0:2 * p1], b.ft_prompt_lens[2 * p0:2 * p1],
               (seg[base + 2 * p0:base + 2 * p1 + 1] - o0).astype(np.int32), b.positions[o0:o1], b.token_ids[o0:o1],
               b.block_size, 4, [], np.full((0, 1), -1, dtype=np.int32), 1)
    return dataclasses.replace(wl, batch=nb, x=wl.x[o0:o1], ctx_k=None, ctx_v=None, ref_logp=wl.ref_logp[2 * p0:2 * p1],
                               pre_k=None, pre_v=None)


def make_upstream_grad(spec: ConfigSpec, n_rows: int, scale: float = 1e-3) -> np.ndarray:
    """A synthetic dL/dY for tests that drive the layer backward on its own."""
    m = spec.dims
    return _maybe_bf16(scale * normal(spec.seed, STREAMS["dy"], 0, n_rows * m.d_model).reshape(n_rows, m.d_model), m.io_bf16)
