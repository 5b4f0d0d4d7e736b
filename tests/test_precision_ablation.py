"""Which contractions of the fine-tune forward need two-term bf16 operands?  (CPU, numpy.)

The HIP path runs every contraction of the fine-tune rows with activations held as two bf16 terms
(hi + lo, about 16 significand bits) so that the DPO loss of Section 3.1 meets |loss - oracle| <= 1e-3
with a margin of five.  This test emulates that operand precision in fp64 numpy - the oracle's
functions for everything that is not a contraction, and for each contraction the rounding the kernels
apply to its operands - and ablates it contraction by contraction: with ONE of them reduced to plain
bf16 operands, how far do the sequence log-probabilities move?

The quantity compared is beta * |d(log p+ - log p-)| per pair, the bound on a pair's loss error for
any reference log-probabilities (|dL/dz| <= 1), next to the loss error itself; a pair whose loss is
saturated hides a log-probability error that another set of reference values would expose.

Result (asserted below): no contraction can take plain bf16 operands at a margin of five - each one
alone moves a pair by 6e-4 to 1e-2 (edge-size pairs) - while the form the library runs (all two-term; the LM head in
one pass plus the first-order term of the dropped lo part) stays under 2e-4."""
import numpy as np
import pytest

from oracle import mace_oracle as O
from paper_2510_03283_amd import synth

MARGIN_BAR = 2e-4     # 1e-3 / 5
CONTRACTIONS = ("q_proj", "k_proj", "v_proj", "qk", "pv", "o", "gate_up", "down")


def _bf(x):
    return synth.round_to_bf16(np.asarray(x, np.float32)).astype(np.float64)


def _f32(x):
    return np.asarray(x, np.float64).astype(np.float32).astype(np.float64)


def _mm(x, W, single):
    """x W^T with x rounded to bf16 (single) or held as hi + lo (two passes); W is bf16 already."""
    hi = _bf(x)
    return hi @ W.T if single else hi @ W.T + _bf(x - hi) @ W.T


def emulated_logp(wl, single=(), head="taylor"):
    """Sequence log-probabilities with the operand rounding of the HIP path.  single: contractions run
    with plain bf16 operands.  head: 'two' (two passes), 'one' (one pass, nothing added back) or
    'taylor' (one pass + n_lo . (dlogits E), what the library runs when gradients are requested)."""
    m, b = wl.dims, wl.batch
    W = {k: np.asarray(v, np.float64) for k, v in wl.weights.items()}
    seg = b.seg_offsets
    grp = m.n_q_heads // m.n_kv_heads
    out = []
    for s in range(len(b.ft_lens)):
        o0, o1 = int(seg[s]), int(seg[s + 1])
        L = o1 - o0
        x = wl.x[o0:o1].astype(np.float64)
        pos = b.positions[o0:o1]
        a, _ = O.rmsnorm(x, W["g1"], m.rms_eps)
        q = O.rope(_f32(_mm(a, W["wq"], "q_proj" in single)).reshape(L, m.n_q_heads, m.head_dim), pos, m.rope_theta)
        k = O.rope(_f32(_mm(a, W["wk"], "k_proj" in single)).reshape(L, m.n_kv_heads, m.head_dim), pos, m.rope_theta)
        v = _f32(_mm(a, W["wv"], "v_proj" in single)).reshape(L, m.n_kv_heads, m.head_dim)
        mask = np.tril(np.ones((L, L), bool))
        o = np.empty((L, m.n_q_heads, m.head_dim))
        for h in range(m.n_q_heads):
            qq, kk, vv = q[:, h], k[:, h // grp], v[:, h // grp]
            qh, kh, vh = _bf(qq), _bf(kk), _bf(vv)
            sc = qh @ kh.T
            if "qk" not in single:
                sc = sc + _bf(qq - qh) @ kh.T + qh @ _bf(kk - kh).T
            sc = np.where(mask, sc / np.sqrt(m.head_dim), -np.inf)
            e = np.exp(sc - sc.max(1, keepdims=True))
            eh = _bf(e)
            pv = eh @ vh
            if "pv" not in single:
                pv = pv + _bf(e - eh) @ vh + eh @ _bf(vv - vh)
            o[:, h] = pv / e.sum(1, keepdims=True)
        x1 = _f32(x + _mm(_f32(o.reshape(L, -1)), W["wo"], "o" in single))
        bb, _ = O.rmsnorm(x1, W["g2"], m.rms_eps)
        hm = O.silu(_f32(_mm(bb, W["wg"], "gate_up" in single))) * _f32(_mm(bb, W["wu"], "gate_up" in single))
        y = _f32(x1 + _mm(hm, W["wd"], "down" in single))
        rows = np.arange(b.ft_prompt_lens[s] - 1, L - 1)
        n, _ = O.rmsnorm(y[rows], W["gf"], m.rms_eps)
        lab = b.token_ids[o0:o1][rows + 1]
        ar = np.arange(len(rows))
        if head == "two":
            lg = _f32(_mm(n, W["E"], False))
            lp = lg[ar, lab] - O.logsumexp(lg, 1)
        else:
            hi = _bf(n)
            lg = _f32(hi @ W["E"].T)
            lse = O.logsumexp(lg, 1)
            lp = lg[ar, lab] - lse
            if head == "taylor":
                dl = -np.exp(lg - lse[:, None])
                dl[ar, lab] += 1.0
                lp = lp + (_bf(n - hi) * (_bf(dl) @ W["E"])).sum(1)
        out.append(float(lp.sum()))
    return np.array(out)


def _errors(wl, lp, lp0):
    loss, loss0 = O.dpo_pair_loss(lp, wl.ref_logp, wl.beta), O.dpo_pair_loss(lp0, wl.ref_logp, wl.beta)
    d_clpd = np.abs((lp[0::2] - lp[1::2]) - (lp0[0::2] - lp0[1::2])).max()
    return float(np.abs(loss[0] - loss0[0]).max()), float(wl.beta * d_clpd)


@pytest.fixture(scope="module")
def edge_pairs():
    wl = synth.make_workload("edge", n_prefill=0, n_decode=0, n_pairs=2, with_cache=False)
    m, b = wl.dims, wl.batch
    ck = O.new_cache(1, m.n_kv_heads, b.block_size, m.head_dim)
    exact = O.hybrid_iteration(m, wl.weights, b, wl.x, ck, ck.copy(), wl.ref_logp, wl.beta, backward=False)
    return wl, np.asarray(exact["head"]["logp"], np.float64)


def test_the_form_the_library_runs_keeps_a_margin_of_five(edge_pairs):
    wl, lp0 = edge_pairs
    for head in ("taylor", "two"):
        dloss, bound = _errors(wl, emulated_logp(wl, head=head), lp0)
        print(f"all two-term, head {head}: worst pair |dloss| {dloss:.2e}, beta |d clpd| {bound:.2e}")
        assert dloss <= MARGIN_BAR and bound <= MARGIN_BAR, (head, dloss, bound)


def test_one_pass_head_needs_its_first_order_term(edge_pairs):
    wl, lp0 = edge_pairs
    _, bound = _errors(wl, emulated_logp(wl, head="one"), lp0)
    print(f"head in one pass, nothing added back: beta |d clpd| {bound:.2e}")
    assert bound > MARGIN_BAR


@pytest.mark.parametrize("c", CONTRACTIONS)
def test_no_contraction_can_drop_its_second_term(edge_pairs, c):
    wl, lp0 = edge_pairs
    dloss, bound = _errors(wl, emulated_logp(wl, single=(c,), head="two"), lp0)
    print(f"plain bf16 operands in {c} alone: worst pair |dloss| {dloss:.2e}, beta |d clpd| {bound:.2e}")
    assert bound > MARGIN_BAR, (c, bound)
