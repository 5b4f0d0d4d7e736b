"""Pins of the oracle's shared-prompt DPO layout (a pair stored once as prompt | chosen | rejected,
both responses attending to one copy of the prompt): it must be the SAME function of the weights
as the two-sequence layout, whose backward has its own finite-difference pins."""
import types

import numpy as np

from oracle import mace_oracle as O
from test_oracle_pins import make_small_batch, rand_weights, small_dims


def _shared_from(b, x):
    """Re-lay a small two-sequence batch (ft only) as shared-prompt pairs."""
    seg = b.seg_offsets
    n_pairs = len(b.ft_lens) // 2
    rows, pos, lens, chosen, prompts = [], [], [], [], []
    for i in range(n_pairs):
        o0, o1, o2 = int(seg[2 * i]), int(seg[2 * i + 1]), int(seg[2 * i + 2])
        P = int(b.ft_prompt_lens[2 * i])
        rows += list(range(o0, o1)) + list(range(o1 + P, o2))
        Rc, Rr = o1 - o0 - P, o2 - o1 - P
        pos += list(range(P + Rc)) + list(range(P, P + Rr))
        lens.append(P + Rc + Rr); chosen.append(Rc); prompts.append(P)
    rows = np.array(rows)
    sb = types.SimpleNamespace(**vars(b))
    sb.ft_lens = np.array(lens); sb.ft_prompt_lens = np.array(prompts); sb.ft_chosen_lens = np.array(chosen)
    sb.seg_offsets = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    sb.positions = np.array(pos, np.int32); sb.token_ids = b.token_ids[rows]
    return sb, x[rows], rows


def test_shared_prompt_equals_two_sequence_layout():
    rng = np.random.default_rng(41)
    m = small_dims(Hq=4, Hkv=2)
    W = rand_weights(m, rng, scale=0.3)
    b = make_small_batch(m, rng, prefill=(), decode=(), ft=((3, 4), (3, 2), (2, 3), (2, 5)))
    seg = b.seg_offsets
    # the two sequences of a pair share their prompt tokens (and so their prompt rows of x)
    T = int(seg[-1])
    x = rng.normal(size=(T, m.d_model))
    for i in range(2):
        P = int(b.ft_prompt_lens[2 * i])
        x[seg[2 * i + 1]:seg[2 * i + 1] + P] = x[seg[2 * i]:seg[2 * i] + P]
        b.token_ids[seg[2 * i + 1]:seg[2 * i + 1] + P] = b.token_ids[seg[2 * i]:seg[2 * i] + P]
    ref = rng.normal(-8, 1, 4); beta = 0.4
    ck = O.new_cache(b.num_blocks, m.n_kv_heads, b.block_size, m.head_dim)
    A = O.hybrid_iteration(m, W, b, x, ck.copy(), ck.copy(), ref, beta)
    sb, xs, rows = _shared_from(b, x)
    S = O.hybrid_iteration(m, W, sb, xs, ck.copy(), ck.copy(), ref, beta)
    assert np.allclose(S["head"]["logp"], A["head"]["logp"], rtol=1e-12)
    assert np.allclose(S["head"]["loss_per_pair"], A["head"]["loss_per_pair"], rtol=1e-12)
    assert np.array_equal(S["head"]["win"], A["head"]["win"])
    assert np.allclose(S["y"], A["y"][rows], rtol=1e-11, atol=1e-13)              # the kept rows are the same rows
    for k in A["grads"]:
        assert np.allclose(S["grads"][k], A["grads"][k], rtol=1e-9, atol=1e-13), k  # same function of the weights
    # dx: response rows as before; a prompt row collects the gradient of its two copies
    want = A["dx_ft"][rows].copy()
    off = 0
    for i in range(2):
        P = int(b.ft_prompt_lens[2 * i])
        want[off:off + P] += A["dx_ft"][seg[2 * i + 1]:seg[2 * i + 1] + P]
        off += int(sb.ft_lens[i])
    assert np.allclose(S["dx_ft"], want, rtol=1e-9, atol=1e-13)
    # the excluded rectangle is really excluded: the rejected rows' probabilities on chosen keys are zero
    P0, Rc0 = int(sb.ft_prompt_lens[0]), int(sb.ft_chosen_lens[0])
    Pm = S["saved"][0]["P"]
    assert np.all(Pm[:, P0 + Rc0:, P0:P0 + Rc0] == 0) and np.all(Pm[:, P0 + Rc0:, :P0] > 0)


def test_attention_excluded_rectangle_brute_force():
    rng = np.random.default_rng(42)
    L, lo, hi = 9, 3, 6
    q = rng.normal(size=(L, 2, 4)); k = rng.normal(size=(L, 1, 4)); v = rng.normal(size=(L, 1, 4))
    o, lse, P = O.causal_attention(q, k, v, (lo, hi))
    for h in range(2):
        for t in range(L):
            keys = [j for j in range(t + 1) if not (t >= hi and lo <= j < hi)]
            s = np.array([q[t, h] @ k[j, 0] / 2.0 for j in keys])
            w = np.exp(s - s.max()); w /= w.sum()
            assert np.allclose(o[t, h], sum(wj * v[j, 0] for wj, j in zip(w, keys)), atol=1e-12)
            assert np.isclose(lse[t, h], s.max() + np.log(np.exp(s - s.max()).sum()))
