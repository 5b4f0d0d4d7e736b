"""Pins of the oracle's cache-pruning statistics (Section 4.3): head norms of decode rows, their
running mean, the per-head capacity split and the prune predicate."""
import numpy as np

from oracle import mace_oracle as O
from test_oracle_pins import make_small_batch, rand_weights, small_dims


def test_head_norm_of_a_one_key_context_is_the_value_norm():
    """A decode row with no cached context attends to itself only: the output of head h is its own
    value row of the kv head h // group, whatever q and k are."""
    rng = np.random.default_rng(3)
    m = small_dims(Hq=4, Hkv=2)
    W = rand_weights(m, rng)
    b = make_small_batch(m, rng, prefill=(), decode=(0, 5), ft=())
    T = int(b.seg_offsets[-1])
    x = rng.normal(size=(T, m.d_model))
    ck = rng.normal(size=(b.num_blocks, m.n_kv_heads, b.block_size, m.head_dim))
    cv = rng.normal(size=ck.shape)
    ex = {}
    O.layer_forward(m, W, b, x, ck, cv, extras=ex)
    hn = ex["head_norms"]
    assert hn.shape == (2, m.n_q_heads)
    a, _ = O.rmsnorm(x[0:1], W["g1"], m.rms_eps)
    v = (a @ W["wv"].T).reshape(m.n_kv_heads, m.head_dim)
    want = np.linalg.norm(v, axis=-1)[np.arange(m.n_q_heads) // (m.n_q_heads // m.n_kv_heads)]
    assert np.allclose(hn[0], want, rtol=1e-12)
    # a convex combination of value rows can not be longer than the longest of them
    K, _ = O.kv_gather(ck, b.decode_block_tables[1], 6)
    V, _ = O.kv_gather(cv, b.decode_block_tables[1], 6)
    vmax = np.linalg.norm(np.asarray(V), axis=-1).max(axis=0)          # per kv head
    assert np.all(hn[1] <= vmax[np.arange(m.n_q_heads) // 2] + 1e-12)


def test_running_mean_is_the_arithmetic_mean():
    rng = np.random.default_rng(4)
    seq = rng.uniform(0.1, 3.0, size=(7, 3, 5))       # 7 iterations, 3 requests, 5 heads
    abar = np.zeros((3, 5))
    for t in range(7):
        abar = O.rolling_mean_update(abar, seq[t], np.full(3, t + 1))
        assert np.allclose(abar, seq[:t + 1].mean(axis=0), rtol=1e-13)
    # requests at different iteration counts
    abar = np.array([[2.0, 4.0], [1.0, 1.0]])
    out = O.rolling_mean_update(abar, np.array([[4.0, 4.0], [3.0, 0.0]]), np.array([2, 4]))
    assert np.allclose(out, [[3.0, 4.0], [1.5, 0.75]])


def test_head_budget_worked_examples_and_invariants():
    assert list(O.head_budget([1.0, 1.0, 2.0], 10)) == [2, 2, 6]          # floors 2,2,5 -> one left -> largest weight
    assert list(O.head_budget([1.0, 1.0, 1.0], 10)) == [4, 3, 3]          # tie: lower index first
    assert list(O.head_budget([3.0, 1.0], 8)) == [6, 2]                   # exact split, nothing left
    assert list(O.head_budget([0.5, 0.25, 0.25], 1)) == [1, 0, 0]
    assert list(O.head_budget([5.0], 17)) == [17]
    rng = np.random.default_rng(6)
    for _ in range(200):
        H = int(rng.integers(1, 33))
        abar = rng.uniform(0.01, 5.0, H)
        C = int(rng.integers(0, 100000))
        c = O.head_budget(abar, C)
        w = abar / abar.sum()
        assert c.sum() == C and np.all(c >= np.floor(w * C)) and np.all(c <= np.floor(w * C) + 1)
        # monotone: a head with a strictly larger weight never gets less
        o = np.argsort(w)
        assert np.all(np.diff(c[o]) >= 0) or np.all(c[o][1:] + 1 >= c[o][:-1])
    assert list(O.head_budget(2.0 * np.array([1.0, 1.0, 2.0]), 10)) == [2, 2, 6]      # scale invariant


def test_prune_predicate():
    norms = np.array([[0.5, 2.0, 2.0], [0.1, 0.1, 3.0]])
    last = np.array([[9, 9, 2], [7, 1, 7]])
    flags, new_last = O.prune_flags(norms, t_now=[10, 8], t_last_used=last, window=4, tau=1.0)
    # request 0: head 0 low norm -> prune; head 1 fine; head 2 norm fine but idle for 8 > 4 -> prune
    assert flags.tolist() == [[True, False, True], [True, True, False]]
    assert new_last.tolist() == [[9, 10, 10], [7, 1, 8]]
