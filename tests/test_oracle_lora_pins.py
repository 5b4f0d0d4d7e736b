"""Pins of the oracle's adapter (LoRA) path against things other than itself: the base model
(B = 0), the merged weight W + scale*B*A run through the FULL-weight path (which has its own
finite-difference pins), and central finite differences on adapter entries."""
import numpy as np

from oracle import mace_oracle as O
from test_oracle_pins import make_small_batch, rand_weights, small_dims


def rand_lora(m, rng, rank=3, scale=1.7, sigma=0.3):
    qd, kvd = m.n_q_heads * m.head_dim, m.n_kv_heads * m.head_dim
    io = {"q": (qd, m.d_model), "k": (kvd, m.d_model), "v": (kvd, m.d_model), "o": (m.d_model, qd)}
    lora = {"rank": rank, "scale": scale}
    for p, (n_out, n_in) in io.items():
        lora["a_" + p] = rng.normal(0, sigma, (rank, n_in))
        lora["b_" + p] = rng.normal(0, sigma, (n_out, rank))
    return lora


def merged(W, lora):
    Wm = dict(W)
    for p, wn in (("q", "wq"), ("k", "wk"), ("v", "wv"), ("o", "wo")):
        Wm[wn] = W[wn] + lora["scale"] * (lora["b_" + p] @ lora["a_" + p])
    return Wm


def setup(seed=5, with_inference=True):
    rng = np.random.default_rng(seed)
    m = small_dims(Hq=4, Hkv=2)
    W = rand_weights(m, rng, scale=0.3)
    if with_inference:
        b = make_small_batch(m, rng, ft=((3, 4), (3, 2), (2, 3), (2, 3)))
    else:
        b = make_small_batch(m, rng, prefill=(), decode=(), ft=((3, 4), (3, 2), (2, 3), (2, 3)))
    T = int(b.seg_offsets[-1])
    x = rng.normal(size=(T, m.d_model))
    ref = rng.normal(-8, 1, 4)
    lora = rand_lora(m, rng)
    return rng, m, W, b, x, ref, lora


def run(m, W, b, x, ref, beta, lora, rng_cache_seed=11):
    rng = np.random.default_rng(rng_cache_seed)
    ck = rng.normal(size=(b.num_blocks, m.n_kv_heads, b.block_size, m.head_dim))
    cv = rng.normal(size=ck.shape)
    return O.hybrid_iteration(m, W, b, x, ck, cv, ref, beta, lora=lora), ck, cv


def test_zero_b_is_the_base_model():
    rng, m, W, b, x, ref, lora = setup()
    z = dict(lora)
    for p in "qkvo":
        z["b_" + p] = np.zeros_like(lora["b_" + p])
    a, cka, cva = run(m, W, b, x, ref, 0.4, z)
    base, ckb, cvb = run(m, W, b, x, ref, 0.4, None)
    assert np.array_equal(a["y"], base["y"]) and np.array_equal(cka, ckb) and np.array_equal(cva, cvb)
    assert np.array_equal(a["head"]["loss_per_pair"], base["head"]["loss_per_pair"])
    assert np.allclose(a["dx_ft"], base["dx_ft"], atol=1e-14)
    # with B = 0 nothing flows into A, and dB = scale * dW A^T of the base model
    for p, wn in (("q", "wq"), ("k", "wk"), ("v", "wv"), ("o", "wo")):
        assert np.all(a["grads"]["a_" + p] == 0)
        assert np.allclose(a["grads"]["b_" + p], z["scale"] * base["grads"][wn] @ z["a_" + p].T, rtol=1e-10, atol=1e-13)


def test_adapter_equals_merged_weight():
    rng, m, W, b, x, ref, lora = setup()
    a, cka, cva = run(m, W, b, x, ref, 0.4, lora)
    f, ckf, cvf = run(m, merged(W, lora), b, x, ref, 0.4, None)       # full-weight path, independent pins
    assert np.allclose(a["y"], f["y"], rtol=1e-11, atol=1e-12)
    assert np.allclose(cka, ckf, rtol=1e-11, atol=1e-12) and np.allclose(cva, cvf, rtol=1e-11, atol=1e-12)
    assert np.array_equal(a["slots"], f["slots"])
    assert np.allclose(a["head"]["logp"], f["head"]["logp"], rtol=1e-11)
    assert np.allclose(a["head"]["loss_per_pair"], f["head"]["loss_per_pair"], rtol=1e-10)
    assert np.allclose(a["dx_ft"], f["dx_ft"], rtol=1e-9, atol=1e-13)
    # chain rule through W' = W + s B A:  dA = s B^T dW',  dB = s dW' A^T
    s = lora["scale"]
    for p, wn in (("q", "wq"), ("k", "wk"), ("v", "wv"), ("o", "wo")):
        dW = f["grads"][wn]
        assert np.allclose(a["grads"]["a_" + p], s * lora["b_" + p].T @ dW, rtol=1e-9, atol=1e-13), p
        assert np.allclose(a["grads"]["b_" + p], s * dW @ lora["a_" + p].T, rtol=1e-9, atol=1e-13), p
    assert set(a["grads"]) == {x + y for x in ("a_", "b_") for y in "qkvo"}     # nothing else is trained


def test_adapter_gradients_match_central_differences():
    rng, m, W, b, x, ref, lora = setup(seed=9, with_inference=False)
    beta = 0.4
    ck = O.new_cache(b.num_blocks, m.n_kv_heads, b.block_size, m.head_dim)

    def loss(l):
        return O.hybrid_iteration(m, W, b, x, ck.copy(), ck.copy(), ref, beta, backward=False, lora=l)["head"]["loss_mean"]

    out = O.hybrid_iteration(m, W, b, x, ck.copy(), ck.copy(), ref, beta, lora=lora)
    h = 1e-5
    for name in [x + y for x in ("a_", "b_") for y in "qkvo"]:
        for _ in range(4):
            idx = tuple(rng.integers(0, s) for s in lora[name].shape)
            lp = dict(lora); lp[name] = lora[name].copy(); lp[name][idx] += h
            lm = dict(lora); lm[name] = lora[name].copy(); lm[name][idx] -= h
            fd = (loss(lp) - loss(lm)) / (2 * h)
            assert abs(fd - out["grads"][name][idx]) <= 1e-6 * max(1.0, abs(fd)) + 1e-9, (name, idx, fd)
        D = rng.normal(size=lora[name].shape)
        lp = dict(lora); lp[name] = lora[name] + h * D
        lm = dict(lora); lm[name] = lora[name] - h * D
        fd = (loss(lp) - loss(lm)) / (2 * h)
        an = float(np.sum(D * out["grads"][name]))
        assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, fd, an)
    # scale enters linearly in the adapter term: doubling scale and halving B changes nothing
    l2 = dict(lora); l2["scale"] = 2 * lora["scale"]
    for p in "qkvo":
        l2["b_" + p] = lora["b_" + p] / 2
    o2 = O.hybrid_iteration(m, W, b, x, ck.copy(), ck.copy(), ref, beta, lora=l2)
    assert np.allclose(o2["y"], out["y"], rtol=1e-12) and np.allclose(o2["grads"]["a_q"], out["grads"]["a_q"], rtol=1e-10)
    assert np.allclose(o2["grads"]["b_o"], 2 * out["grads"]["b_o"], rtol=1e-10)
