"""Pins of the two oracle functions that close the serving / training loop: next-token logits of
inference rows and the AdamW step."""
import numpy as np

from oracle import mace_oracle as O
from test_oracle_pins import rand_weights, small_dims


def test_next_token_logits_closed_forms():
    rng = np.random.default_rng(31)
    m = small_dims()
    W = rand_weights(m, rng)
    y = rng.normal(size=(5, m.d_model))
    logits, nxt = O.next_token_logits(m, W, y)
    # the same rows through the sequence log-prob path (pinned elsewhere): logits agree
    _, sv = O.sequence_logprob(m, W, np.concatenate([y, y[:1]]), np.zeros(6, np.int64), 1)
    assert np.allclose(logits, sv["logits"], atol=1e-13)
    # scale invariance of the final RMSNorm: the logits do not change when a row is rescaled
    l2, n2 = O.next_token_logits(m, W, 7.5 * y)
    assert np.allclose(l2, logits, rtol=1e-5, atol=1e-8) and np.array_equal(n2, nxt)     # exact up to eps in the norm
    # a row aligned with g_f-weighted embedding v picks token v
    for tok in (0, 7, m.vocab - 1):
        row = W["E"][tok] / W["gf"]                      # RMSNorm then * g_f gives a multiple of E[tok]
        l, a = O.next_token_logits(m, W, row[None, :])
        c = W["E"] @ W["E"][tok]
        assert a[0] == int(np.argmax(c))                 # argmax of E E[tok]^T, which is tok unless another row is longer
    # ties go to the lowest index
    Wt = dict(W); Wt["E"] = W["E"].copy(); Wt["E"][3] = Wt["E"][1]
    l, a = O.next_token_logits(m, Wt, y)
    assert np.all(a != 3)


def test_adamw_closed_forms():
    rng = np.random.default_rng(32)
    p = rng.normal(size=50); g = rng.normal(size=50)
    lr, b1, b2, eps, wd = 1e-2, 0.9, 0.999, 1e-8, 0.1
    # first step from zero moments: mhat = g, vhat = g^2  ->  p - lr (g / (|g| + eps) + wd p)
    p1, m1, v1 = O.adamw_step(p, g, np.zeros(50), np.zeros(50), 1, lr, b1, b2, eps, wd)
    assert np.allclose(m1, 0.1 * g) and np.allclose(v1, 0.001 * g * g)
    assert np.allclose(p1, p - lr * (g / (np.abs(g) + eps) + wd * p), rtol=1e-12)
    # zero gradient and zero moments: pure decay
    p2, m2, v2 = O.adamw_step(p, np.zeros(50), np.zeros(50), np.zeros(50), 1, lr, b1, b2, eps, wd)
    assert np.allclose(p2, p * (1 - lr * wd)) and np.all(m2 == 0) and np.all(v2 == 0)
    # no decay, constant gradient: every step moves by lr * sign(g) (bias correction makes mhat = g, vhat = g^2)
    q, m, v = p.copy(), np.zeros(50), np.zeros(50)
    for t in range(1, 6):
        q, m, v = O.adamw_step(q, g, m, v, t, lr, b1, b2, 0.0, 0.0)
    assert np.allclose(q, p - 5 * lr * np.sign(g), rtol=1e-10)


def test_adamw_matches_torch_on_cpu():
    import torch
    rng = np.random.default_rng(33)
    p0 = rng.normal(size=(7, 9)); lr, b1, b2, eps, wd = 3e-3, 0.8, 0.95, 1e-6, 0.05
    tp = torch.nn.Parameter(torch.tensor(p0, dtype=torch.float64))
    opt = torch.optim.AdamW([tp], lr=lr, betas=(b1, b2), eps=eps, weight_decay=wd)
    p, m, v = p0.copy(), np.zeros_like(p0), np.zeros_like(p0)
    for t in range(1, 5):
        g = rng.normal(size=p0.shape)
        tp.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        p, m, v = O.adamw_step(p, g, m, v, t, lr, b1, b2, eps, wd)
        # torch adds eps after dividing sqrt(v) by sqrt(1 - b2^t): the same formula
        assert np.allclose(p, tp.detach().numpy(), rtol=1e-10, atol=1e-13), t
