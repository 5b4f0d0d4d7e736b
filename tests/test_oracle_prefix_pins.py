"""Pins of the oracle's prefix-shared prefill (Section 4.3, "Reduced prefill via prefix tree"):
a request whose first P tokens are cached must give, for its new rows, exactly what a one-piece
prefill of the whole sequence gives for those rows - attention is causal, so the prefix rows do
not depend on what follows them."""
import copy
import math
import types

import numpy as np

from oracle import mace_oracle as O
from test_oracle_pins import make_small_batch, rand_weights, small_dims


def brute_prefix_attention(q, K, V, P):
    L, Hq, hd = q.shape
    grp = Hq // K.shape[1]
    o = np.zeros((L, Hq, hd))
    for h in range(Hq):
        for j in range(L):
            s = [sum(q[j, h, e] * K[t, h // grp, e] for e in range(hd)) / math.sqrt(hd) for t in range(P + j + 1)]
            mx = max(s)
            w = [math.exp(a - mx) for a in s]
            z = sum(w)
            for t in range(P + j + 1):
                o[j, h] += w[t] / z * V[t, h // grp]
    return o


def test_prefix_attention_brute_force_and_zero_prefix():
    rng = np.random.default_rng(21)
    q = rng.normal(size=(5, 4, 8)); K = rng.normal(size=(12, 2, 8)); V = rng.normal(size=(12, 2, 8))
    assert np.allclose(O.prefix_causal_attention(q, K, V, 7), brute_prefix_attention(q, K, V, 7), atol=1e-12)
    o0, _, _ = O.causal_attention(q, K[:5], V[:5])
    assert np.allclose(O.prefix_causal_attention(q, K[:5], V[:5], 0), o0, atol=1e-13)
    # a prefix whose keys score -inf-like low leaves the plain causal result (softmax weight -> 0)
    Kfar = K.copy(); Kfar[:7] = -1e3 * np.sign(q.mean(axis=(0, 1)))[None, None, :] * np.ones((7, 2, 8))
    # (only a smoke property: result stays finite and rows are convex combinations of V)
    o = O.prefix_causal_attention(q, Kfar, V, 7)
    assert np.all(np.isfinite(o)) and np.all(np.abs(o) <= np.abs(V).max() + 1e-12)


def _one_request_batch(m, rng, tokens_pos0, L, P, B, table):
    seg = np.array([0, L], np.int32)
    return types.SimpleNamespace(prefill_lens=np.array([L]), decode_ctx=np.array([], np.int64), ft_lens=np.array([], np.int64),
                                 ft_prompt_lens=np.array([], np.int64), seg_offsets=seg,
                                 positions=(np.arange(L) + P).astype(np.int32), token_ids=tokens_pos0, block_size=B,
                                 num_blocks=0, prefill_block_tables=[table], decode_block_tables=np.zeros((0, 1), np.int32),
                                 prefill_prefix_lens=np.array([P]))


def test_prefix_prefill_equals_tail_of_whole_prefill_and_blocks_can_be_shared():
    rng = np.random.default_rng(22)
    m = small_dims(Hq=4, Hkv=2)
    W = rand_weights(m, rng)
    B, P, L1, L2 = 4, 8, 5, 7               # the prefix fills two whole blocks, so two requests can share them
    nblk = 12
    x_prefix = rng.normal(size=(P, m.d_model))
    x1 = rng.normal(size=(L1, m.d_model)); x2 = rng.normal(size=(L2, m.d_model))
    shared = np.array([9, 2], np.int32)
    t1 = np.concatenate([shared, [5, 0]]).astype(np.int32)      # ceil((8+5)/4) = 4 blocks
    t2 = np.concatenate([shared, [7, 3]]).astype(np.int32)      # ceil((8+7)/4) = 4 blocks
    # reference: each whole sequence prefilled in one piece into its own fresh cache
    def whole(xs, table):
        ck = np.zeros((nblk, m.n_kv_heads, B, m.head_dim)); cv = np.zeros_like(ck)
        b = _one_request_batch(m, rng, None, len(xs), 0, B, table)
        y, _, _ = O.layer_forward(m, W, b, xs, ck, cv)
        return y, ck, cv
    y1w, ck1, cv1 = whole(np.concatenate([x_prefix, x1]), t1)
    y2w, ck2, cv2 = whole(np.concatenate([x_prefix, x2]), t2)
    # prefix-shared: the prefix is prefilled once into the shared blocks, then both requests run in ONE batch
    ck = np.zeros((nblk, m.n_kv_heads, B, m.head_dim)); cv = np.zeros_like(ck)
    bp = _one_request_batch(m, rng, None, P, 0, B, shared)
    yp, _, _ = O.layer_forward(m, W, bp, x_prefix, ck, cv)
    assert np.allclose(yp, y1w[:P], atol=1e-12)                  # causal: prefix rows do not see what follows
    b = types.SimpleNamespace(prefill_lens=np.array([L1, L2]), decode_ctx=np.array([], np.int64), ft_lens=np.array([], np.int64),
                              ft_prompt_lens=np.array([], np.int64), seg_offsets=np.array([0, L1, L1 + L2], np.int32),
                              positions=np.concatenate([np.arange(L1) + P, np.arange(L2) + P]).astype(np.int32), token_ids=None,
                              block_size=B, num_blocks=nblk, prefill_block_tables=[t1, t2],
                              decode_block_tables=np.zeros((0, 1), np.int32), prefill_prefix_lens=np.array([P, P]))
    y, slots, _ = O.layer_forward(m, W, b, np.concatenate([x1, x2]), ck, cv)
    assert np.allclose(y[:L1], y1w[P:], atol=1e-12) and np.allclose(y[L1:], y2w[P:], atol=1e-12)
    # the new rows landed behind the prefix, in each request's own blocks; the shared blocks are untouched
    assert np.array_equal(slots[:L1], O.slot_mapping(t1, B, P, L1)) and np.array_equal(slots[L1:], O.slot_mapping(t2, B, P, L2))
    for blk in (5, 0):
        assert np.allclose(ck[blk], ck1[blk], atol=1e-12) and np.allclose(cv[blk], cv1[blk], atol=1e-12)
    for blk in (7, 3):
        assert np.allclose(ck[blk], ck2[blk], atol=1e-12)
    for blk in shared:
        assert np.allclose(ck[blk], ck1[blk], atol=1e-12) and np.allclose(ck[blk], ck2[blk], atol=1e-12)


def test_prefix_not_on_a_block_boundary():
    """A request may also continue its own partially filled block (chunked prefill): P = 6, B = 4."""
    rng = np.random.default_rng(23)
    m = small_dims(Hq=2, Hkv=2)
    W = rand_weights(m, rng)
    B, P, L = 4, 6, 5
    xs = rng.normal(size=(P + L, m.d_model))
    table = np.array([3, 1, 4], np.int32)
    ckw = np.zeros((6, m.n_kv_heads, B, m.head_dim)); cvw = np.zeros_like(ckw)
    yw, _, _ = O.layer_forward(m, W, _one_request_batch(m, rng, None, P + L, 0, B, table), xs, ckw, cvw)
    ck = np.zeros_like(ckw); cv = np.zeros_like(ckw)
    O.layer_forward(m, W, _one_request_batch(m, rng, None, P, 0, B, table[:2]), xs[:P], ck, cv)
    y, _, _ = O.layer_forward(m, W, _one_request_batch(m, rng, None, L, P, B, table), xs[P:], ck, cv)
    assert np.allclose(y, yw[P:], atol=1e-12) and np.allclose(ck, ckw, atol=1e-12) and np.allclose(cv, cvw, atol=1e-12)
