"""CPU oracle for one hybrid iteration of a pre-norm decoder layer with a DPO head.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain fp64 definition the HIP library is
checked against.  Only the tests, the smoke check and the benchmark's cpu_baseline leg may
import it; the product path never does.  It shares no code with the HIP path and imports
nothing from it.

What it computes follows the paper's problem statement: an iteration whose batch holds
prefill requests, decode requests with a cached context and preference pairs for fine-tuning
side by side (Fig. 1, Section 4), exact attention over a paged KV cache (Section 3.2,
Section 5), and the DPO objective with its alignment metrics (Section 3.1).  Colocation is an
execution strategy: every request's result equals what it would be when run alone, so the
oracle simply walks the requests one by one and applies the textbook definitions.  The layer
arithmetic (RMSNorm, rotary embedding with half-split pairs, grouped-query attention, SwiGLU,
tied LM head behind a final RMSNorm) is that of the Mistral/LLaMA family the paper serves.

All arithmetic is float64 numpy.  `@` (a library matmul) is used as a step; there is no
tiling, fusion or reordering.  Backward formulas are written out by hand (no autodiff).

Pins (tests/test_oracle_*.py): brute-force soft-max attention, decode == last row of causal
attention, GQA == MHA with repeated KV heads, RoPE identities, RMSNorm scale invariance,
closed forms of the DPO loss, uniform-logit closed form of the LM head, central finite
differences for every gradient, batch-composition invariance, cache round trips; for the
adapter path: zero B == base model, equality with the merged weight W + scale*B*A in the forward
and in dx, dA = scale*B^T dW and dB = scale*dW A^T against the full-weight gradient, and
central finite differences on adapter entries; for the pruning statistics: a one-key context
(the head norm is the norm of that value row), the running mean against the arithmetic mean,
hand-worked capacity splits and their invariants; for prefix-shared prefill: zero prefix ==
plain causal attention, the tail rows of a one-piece prefill of the whole sequence, two
requests sharing the blocks of one prefix, brute force; for the optimizer step: the first-step
closed form, zero gradient, and torch.optim.AdamW on the CPU; for the shared-prompt layout of
a pair: losses, log-probabilities and every weight gradient equal those of the two-sequence
layout, and dx of a prompt row is the sum of its two copies.  The paper
prints no worked numerical example for this path, so absolute values of the benchmark
configurations are pinned by these invariants only.
"""
from __future__ import annotations

import numpy as np

F64 = np.float64


# --------------------------------------------------------------------------- elementary pieces

def rmsnorm(x, g, eps):
    """a = x * (mean_k x_k^2 + eps)^(-1/2) * g, row-wise.  Returns (a, r) with r the row scale."""
    x = np.asarray(x, F64)
    r = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps)
    return x * r * np.asarray(g, F64), r


def rmsnorm_bwd(dy, x, g, r):
    """Gradients of rmsnorm: dg = sum_t dy*x*r ; dx = r*(dy*g) - x*r^3*mean_k((dy*g)*x)."""
    dy, x, g = np.asarray(dy, F64), np.asarray(x, F64), np.asarray(g, F64)
    dg = np.sum(dy * x * r, axis=0)
    u = dy * g
    dx = r * u - x * (r ** 3) * np.mean(u * x, axis=-1, keepdims=True)
    return dx, dg


def rope(u, pos, theta, sign=1.0):
    """Rotary embedding on u[T, H, hd] with half-split pairs (i, i+hd/2), angle pos*theta^(-2i/hd).
    sign=-1 rotates back (the transpose of the rotation, used in the backward pass)."""
    u = np.asarray(u, F64)
    hd = u.shape[-1]
    half = hd // 2
    inv_freq = F64(theta) ** (-2.0 * np.arange(half, dtype=F64) / hd)
    phi = np.asarray(pos, F64)[:, None] * inv_freq[None, :]          # [T, half]
    c, s = np.cos(phi)[:, None, :], sign * np.sin(phi)[:, None, :]
    lo, hi = u[..., :half], u[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def silu(g):
    return g / (1.0 + np.exp(-g))


def sigmoid(g):
    return 1.0 / (1.0 + np.exp(-g))


def logsumexp(l, axis=-1):
    m = np.max(l, axis=axis, keepdims=True)
    return (m + np.log(np.sum(np.exp(l - m), axis=axis, keepdims=True))).squeeze(axis)


# --------------------------------------------------------------------------- paged KV cache

def slot_mapping(block_table, block_size, start_pos, n):
    """Cache slot of positions start_pos .. start_pos+n-1 of one request:
    slot(p) = block_table[p // B] * B + p % B."""
    p = np.arange(start_pos, start_pos + n, dtype=np.int64)
    bt = np.asarray(block_table, dtype=np.int64)
    return bt[p // block_size] * block_size + p % block_size


def cache_element_offset(slot, kvh, e, block_size, n_kv_heads, head_dim):
    """Element offset of (slot, kv head, element) in the layout [blocks, Hkv, B, hd] (int64)."""
    slot = np.asarray(slot, dtype=np.int64)
    return ((slot // block_size) * n_kv_heads + kvh) * block_size * head_dim + (slot % block_size) * head_dim + e


def kv_append(cache, new, slots):
    """Write new[n, Hkv, hd] at `slots` of cache[blocks, Hkv, B, hd]; slot -1 is skipped."""
    B = cache.shape[2]
    for i, s in enumerate(np.asarray(slots, dtype=np.int64)):
        if s < 0:
            continue
        cache[s // B, :, s % B, :] = new[i]


def kv_gather(cache, block_table, ctx_len):
    """Rows of positions 0..ctx_len-1 in order, and their slots."""
    B = cache.shape[2]
    slots = slot_mapping(block_table, B, 0, ctx_len)
    out = np.empty((ctx_len, cache.shape[1], cache.shape[3]), dtype=cache.dtype)
    for p, s in enumerate(slots):
        out[p] = cache[s // B, :, s % B, :]
    return out, slots


# --------------------------------------------------------------------------- attention

def causal_attention(q, k, v, excl=None):
    """Exact causal attention of one sequence.  q[L, Hq, hd], k, v[L, Hkv, hd].
    Query head h uses kv head h // (Hq/Hkv).  Returns o[L, Hq, hd], lse[L, Hq] and the
    probabilities P[Hq, L, L] (kept for the hand-written backward).
    excl = (lo, hi), optional: rows >= hi do not see keys lo .. hi-1.  With the rows of a preference
    pair laid out as prompt | chosen response | rejected response and (lo, hi) = the chosen
    response, both responses attend to ONE copy of the prompt and not to each other."""
    L, Hq, hd = q.shape
    grp = Hq // k.shape[1]
    o = np.empty((L, Hq, hd), F64)
    lse = np.empty((L, Hq), F64)
    P = np.zeros((Hq, L, L), F64)
    mask = np.tril(np.ones((L, L), dtype=bool))
    if excl is not None:
        lo, hi = int(excl[0]), int(excl[1])
        mask[hi:, lo:hi] = False
    for h in range(Hq):
        kh, vh = k[:, h // grp, :], v[:, h // grp, :]
        s = (q[:, h, :] @ kh.T) / np.sqrt(F64(hd))
        s = np.where(mask, s, -np.inf)
        m = np.max(s, axis=1, keepdims=True)
        e = np.exp(s - m)
        z = np.sum(e, axis=1, keepdims=True)
        P[h] = e / z
        o[:, h, :] = P[h] @ vh
        lse[:, h] = (m + np.log(z))[:, 0]
    return o, lse, P


def decode_attention(q, K, V):
    """One query row q[Hq, hd] against all keys K, V[n+1, Hkv, hd] (cached context plus the
    row's own key)."""
    Hq, hd = q.shape
    grp = Hq // K.shape[1]
    o = np.empty((Hq, hd), F64)
    for h in range(Hq):
        s = (K[:, h // grp, :] @ q[h]) / np.sqrt(F64(hd))
        p = np.exp(s - np.max(s))
        p = p / np.sum(p)
        o[h] = p @ V[:, h // grp, :]
    return o


def prefix_causal_attention(q, K, V, n_prefix):
    """Attention of L new rows of a request whose first n_prefix tokens are already cached (prefix
    sharing, Section 4.3: the prefix is prefilled once and its K, V reused by every request below
    that node).  K, V [n_prefix + L, Hkv, hd] hold the cached prefix followed by the new rows;
    new row j (position n_prefix + j) attends to keys 0 .. n_prefix + j."""
    L, Hq, hd = q.shape
    grp = Hq // K.shape[1]
    n = K.shape[0]
    o = np.empty((L, Hq, hd), F64)
    mask = np.arange(n)[None, :] <= (n_prefix + np.arange(L))[:, None]
    for h in range(Hq):
        s = (q[:, h, :] @ K[:, h // grp, :].T) / np.sqrt(F64(hd))
        s = np.where(mask, s, -np.inf)
        e = np.exp(s - np.max(s, axis=1, keepdims=True))
        o[:, h, :] = (e / np.sum(e, axis=1, keepdims=True)) @ V[:, h // grp, :]
    return o


def causal_attention_bwd(do, q, k, v, o, P):
    """D_t = dO_t.O_t ; dV = P^T dO ; dP = dO V^T ; dS = P*(dP - D) ; dQ = dS K / sqrt(hd) ;
    dK = dS^T Q / sqrt(hd); dK, dV summed over the query heads of a group."""
    L, Hq, hd = q.shape
    grp = Hq // k.shape[1]
    dq = np.zeros_like(q, dtype=F64)
    dk = np.zeros_like(k, dtype=F64)
    dv = np.zeros_like(v, dtype=F64)
    sc = 1.0 / np.sqrt(F64(hd))
    for h in range(Hq):
        g = h // grp
        D = np.sum(do[:, h, :] * o[:, h, :], axis=1, keepdims=True)
        dv[:, g, :] += P[h].T @ do[:, h, :]
        dP = do[:, h, :] @ v[:, g, :].T
        dS = P[h] * (dP - D)
        dq[:, h, :] = (dS @ k[:, g, :]) * sc
        dk[:, g, :] += (dS.T @ q[:, h, :]) * sc
    return dq, dk, dv


# --------------------------------------------------------------------------- the layer

def _w(W, name):
    return np.asarray(W[name], F64)


def adapted_linear(u, W, lora, p):
    """u W^T, plus the low-rank adapter term scale * (u A^T) B^T when `lora` holds a_p / b_p
    (Section 5: a frozen base model shared by all requests with a trainable LoRA adapter on the
    attention layers).  A is [rank, in], B is [out, rank]."""
    y = u @ W.T
    if lora is not None:
        A, B = np.asarray(lora["a_" + p], F64), np.asarray(lora["b_" + p], F64)
        y = y + F64(lora["scale"]) * ((u @ A.T) @ B.T)
    return y


def adapted_linear_bwd(dy, u, W, lora, p):
    """Backward of adapted_linear with the base weight frozen: returns du, dA, dB.
    t = u A^T ; dB = scale * dy^T t ; dt = scale * dy B ; dA = dt^T u ; du = dy W + dt A."""
    A, B = np.asarray(lora["a_" + p], F64), np.asarray(lora["b_" + p], F64)
    s = F64(lora["scale"])
    t = u @ A.T
    dB = s * (dy.T @ t)
    dt = s * (dy @ B)
    dA = dt.T @ u
    du = dy @ W + dt @ A
    return du, dA, dB


def project_qkv(dims, W, x, pos, lora=None):
    """Steps 1-3 of the forward: RMSNorm, Q/K/V projections, RoPE on q and k."""
    a, r1 = rmsnorm(x, _w(W, "g1"), dims.rms_eps)
    T = a.shape[0]
    q = adapted_linear(a, _w(W, "wq"), lora, "q").reshape(T, dims.n_q_heads, dims.head_dim)
    k = adapted_linear(a, _w(W, "wk"), lora, "k").reshape(T, dims.n_kv_heads, dims.head_dim)
    v = adapted_linear(a, _w(W, "wv"), lora, "v").reshape(T, dims.n_kv_heads, dims.head_dim)
    q = rope(q, pos, dims.rope_theta)
    k = rope(k, pos, dims.rope_theta)
    return a, r1, q, k, v


def mlp_block(dims, W, x, attn, lora=None):
    """Steps 6-7: x1 = x + Wo attn ; y = x1 + Wd (silu(Wg b) * (Wu b)), b = RMSNorm(x1)."""
    x1 = np.asarray(x, F64) + adapted_linear(attn, _w(W, "wo"), lora, "o")
    b, r2 = rmsnorm(x1, _w(W, "g2"), dims.rms_eps)
    G = b @ _w(W, "wg").T
    U = b @ _w(W, "wu").T
    Hm = silu(G) * U
    y = x1 + Hm @ _w(W, "wd").T
    return y, dict(x1=x1, b=b, r2=r2, G=G, U=U, Hm=Hm)


def layer_forward(dims, W, batch, x, cache_k, cache_v, lora=None, extras=None):
    """One hybrid iteration of the layer, request by request.

    batch: object with prefill_lens, decode_ctx, ft_lens, seg_offsets, positions, block_size,
    prefill_block_tables, decode_block_tables and, optionally, prefill_prefix_lens (tokens of each
    prefill request that are already cached: shared prefix).  x[T, d] rows ordered prefill | decode | ft.
    cache_k / cache_v: [blocks, Hkv, B, hd] float64, updated in place with the post-RoPE keys
    and the values of the prefill and decode rows.
    lora (optional): adapter on the attention projections; every row of the iteration sees the
    same model, base plus adapter.
    extras (optional dict): receives "head_norms" [n_decode, Hq], the L2 norm of every head's
    attention output vector of each decode row (the signal of the cache-pruning policy, Section 4.3).
    Returns y[T, d], the slot mapping of the inference rows (int64), and per ft sequence the
    intermediates the backward pass needs."""
    x = np.asarray(x, F64)
    T, d = x.shape
    y = np.empty((T, d), F64)
    seg = np.asarray(batch.seg_offsets, dtype=np.int64)
    npf, nd = len(batch.prefill_lens), len(batch.decode_ctx)
    B = batch.block_size
    slots_all = []
    # prefill requests: every token attends to its prefix; K, V go to the cache.  With a cached
    # prefix of P tokens the new rows sit at positions P.., are appended behind it, and attend to
    # the cached rows as well.
    prefix = getattr(batch, "prefill_prefix_lens", None)
    for i in range(npf):
        o0, o1 = seg[i], seg[i + 1]
        P = int(prefix[i]) if prefix is not None else 0
        pos = np.asarray(batch.positions[o0:o1])
        a, r1, q, k, v = project_qkv(dims, W, x[o0:o1], pos, lora)
        slots = slot_mapping(batch.prefill_block_tables[i], B, P, o1 - o0)
        kv_append(cache_k, k, slots)
        kv_append(cache_v, v, slots)
        slots_all.append(slots)
        if P == 0:
            o, _, _ = causal_attention(q, k, v)
        else:
            K, _ = kv_gather(cache_k, batch.prefill_block_tables[i], P + o1 - o0)
            V, _ = kv_gather(cache_v, batch.prefill_block_tables[i], P + o1 - o0)
            o = prefix_causal_attention(q, np.asarray(K, F64), np.asarray(V, F64), P)
        y[o0:o1], _ = mlp_block(dims, W, x[o0:o1], o.reshape(o1 - o0, -1), lora)
    # decode requests: one new token at position n, appended, attends to n+1 keys
    for j in range(nd):
        t = seg[npf + j]
        n = int(batch.decode_ctx[j])
        a, r1, q, k, v = project_qkv(dims, W, x[t:t + 1], np.array([n]), lora)
        slots = slot_mapping(batch.decode_block_tables[j], B, n, 1)
        kv_append(cache_k, k, slots)
        kv_append(cache_v, v, slots)
        slots_all.append(slots)
        K, _ = kv_gather(cache_k, batch.decode_block_tables[j], n + 1)
        V, _ = kv_gather(cache_v, batch.decode_block_tables[j], n + 1)
        o = decode_attention(q[0], np.asarray(K, F64), np.asarray(V, F64))
        if extras is not None:
            extras.setdefault("head_norms", []).append(np.sqrt(np.sum(o * o, axis=-1)))
        y[t:t + 1], _ = mlp_block(dims, W, x[t:t + 1], o.reshape(1, -1), lora)
    # fine-tune sequences: causal attention, nothing cached, intermediates kept
    saved = []
    for s in range(len(batch.ft_lens)):
        o0, o1 = seg[npf + nd + s], seg[npf + nd + s + 1]
        pos = np.asarray(batch.positions[o0:o1])
        a, r1, q, k, v = project_qkv(dims, W, x[o0:o1], pos, lora)
        chosen = getattr(batch, "ft_chosen_lens", None)       # shared-prompt layout: prompt | chosen | rejected
        excl = None
        if chosen is not None:
            excl = (int(batch.ft_prompt_lens[s]), int(batch.ft_prompt_lens[s]) + int(chosen[s]))
        o, lse, P = causal_attention(q, k, v, excl)
        y[o0:o1], sv = mlp_block(dims, W, x[o0:o1], o.reshape(o1 - o0, -1), lora)
        sv.update(x=x[o0:o1], a=a, r1=r1, q=q, k=k, v=v, o=o, lse=lse, P=P, pos=pos)
        saved.append(sv)
    slots_cat = np.concatenate(slots_all) if slots_all else np.zeros(0, np.int64)
    if extras is not None:
        extras["head_norms"] = np.array(extras.get("head_norms", [])).reshape(nd, dims.n_q_heads)
    return y, slots_cat, saved


def layer_backward(dims, W, saved, dy_list):
    """Backward of the layer over the fine-tune sequences.  dy_list[s] = dL/dy of sequence s.
    Returns dx per sequence and the summed weight gradients."""
    names = ["wq", "wk", "wv", "wo", "wg", "wu", "wd", "g1", "g2"]
    grads = {n: np.zeros_like(_w(W, n)) for n in names}
    dxs = []
    for sv, dy in zip(saved, dy_list):
        dy = np.asarray(dy, F64)
        L = dy.shape[0]
        # y = x1 + Hm Wd^T
        dHm = dy @ _w(W, "wd")
        grads["wd"] += dy.T @ sv["Hm"]
        dx1 = dy.copy()
        # Hm = silu(G) * U
        sg = sigmoid(sv["G"])
        dU = dHm * (sv["G"] * sg)
        dG = dHm * sv["U"] * sg * (1.0 + sv["G"] * (1.0 - sg))
        # G = b Wg^T, U = b Wu^T
        db = dG @ _w(W, "wg") + dU @ _w(W, "wu")
        grads["wg"] += dG.T @ sv["b"]
        grads["wu"] += dU.T @ sv["b"]
        # b = RMSNorm(x1; g2)
        dxa, dg2 = rmsnorm_bwd(db, sv["x1"], _w(W, "g2"), sv["r2"])
        grads["g2"] += dg2
        dx1 += dxa
        # x1 = x + attn Wo^T
        attn = sv["o"].reshape(L, -1)
        dattn = dx1 @ _w(W, "wo")
        grads["wo"] += dx1.T @ attn
        dx = dx1.copy()
        # attention and RoPE
        dq, dk, dv = causal_attention_bwd(dattn.reshape(sv["o"].shape), sv["q"], sv["k"], sv["v"], sv["o"], sv["P"])
        dq = rope(dq, sv["pos"], dims.rope_theta, sign=-1.0)
        dk = rope(dk, sv["pos"], dims.rope_theta, sign=-1.0)
        dq2, dk2, dv2 = dq.reshape(L, -1), dk.reshape(L, -1), dv.reshape(L, -1)
        da = dq2 @ _w(W, "wq") + dk2 @ _w(W, "wk") + dv2 @ _w(W, "wv")
        grads["wq"] += dq2.T @ sv["a"]
        grads["wk"] += dk2.T @ sv["a"]
        grads["wv"] += dv2.T @ sv["a"]
        # a = RMSNorm(x; g1)
        dxa, dg1 = rmsnorm_bwd(da, sv["x"], _w(W, "g1"), sv["r1"])
        grads["g1"] += dg1
        dx += dxa
        dxs.append(dx)
    return dxs, grads


# --------------------------------------------------------------------------- DPO head

def softplus(t):
    """log(1 + e^t), stable for large |t|."""
    t = np.asarray(t, F64)
    return np.maximum(t, 0.0) + np.log1p(np.exp(-np.abs(t)))


def dpo_pair_loss(logp, ref_logp, beta):
    """Section 3.1: Delta = log pi_theta - log pi_ref per sequence, z = beta (Delta+ - Delta-),
    loss_i = -log sigmoid(z_i) (the quantity that is minimised and thresholded), mean over the
    pairs; CLPD_i = logp+ - logp-, win_i = [CLPD_i > 0].  Sequence 2i is chosen, 2i+1 rejected.
    Also returns dloss_mean/dlogp per sequence."""
    logp, ref = np.asarray(logp, F64), np.asarray(ref_logp, F64)
    n_pairs = len(logp) // 2
    delta = logp - ref
    z = beta * (delta[0::2] - delta[1::2])
    loss = softplus(-z)
    clpd = logp[0::2] - logp[1::2]
    win = (clpd > 0).astype(np.int32)
    c = (sigmoid(z) - 1.0) * beta / n_pairs          # d mean / d logp(chosen); rejected gets -c
    dlogp = np.empty_like(logp)
    dlogp[0::2], dlogp[1::2] = c, -c
    return loss, float(np.mean(loss)), clpd, win, z, dlogp


def sequence_logprob(dims, W, y_seq, token_ids, prompt_len):
    """log pi(response | prompt) of one sequence from the layer output of its rows: rows
    t = P-1 .. L-2 predict token t+1 through the final RMSNorm and the tied head E.
    Returns the sum over the response tokens and what the backward pass needs."""
    L = y_seq.shape[0]
    rows = np.arange(prompt_len - 1, L - 1)
    n, rf = rmsnorm(y_seq[rows], _w(W, "gf"), dims.rms_eps)
    logits = n @ _w(W, "E").T
    lse = logsumexp(logits, axis=1)
    labels = np.asarray(token_ids)[rows + 1]
    logp_t = logits[np.arange(len(rows)), labels] - lse
    return float(np.sum(logp_t)), dict(rows=rows, n=n, rf=rf, logits=logits, lse=lse, labels=labels, logp_t=logp_t)


def dpo_head_forward(dims, W, batch, y_ft_list, ref_logp, beta):
    """y_ft_list[s]: layer output rows of ft sequence s.  Returns per-sequence log-probs, the
    per-pair losses, their mean, CLPD, win flags and intermediates."""
    seg = np.asarray(batch.seg_offsets, dtype=np.int64)
    base = len(batch.prefill_lens) + len(batch.decode_ctx)
    logp, saved = [], []
    for s, y_seq in enumerate(y_ft_list):
        ids = batch.token_ids[seg[base + s]:seg[base + s + 1]]
        lp, sv = sequence_logprob(dims, W, np.asarray(y_seq, F64), ids, int(batch.ft_prompt_lens[s]))
        sv["y"] = np.asarray(y_seq, F64)
        logp.append(lp)
        saved.append(sv)
    logp = np.array(logp, F64)
    loss, loss_mean, clpd, win, z, dlogp = dpo_pair_loss(logp, ref_logp, beta)
    return dict(logp=logp, loss_per_pair=loss, loss_mean=loss_mean, clpd=clpd, win=win, z=z, dlogp=dlogp, saved=saved)


def rows_logprob(dims, W, y_seq, rows, labels):
    """Sum over the given rows of log softmax(E RMSNorm(y_row))[label]: sequence_logprob with the
    rows and their next tokens listed explicitly."""
    rows, labels = np.asarray(rows, np.int64), np.asarray(labels, np.int64)
    n, rf = rmsnorm(y_seq[rows], _w(W, "gf"), dims.rms_eps)
    logits = n @ _w(W, "E").T
    lse = logsumexp(logits, axis=1)
    logp_t = logits[np.arange(len(rows)), labels] - lse
    return float(np.sum(logp_t)), dict(rows=rows, n=n, rf=rf, logits=logits, lse=lse, labels=labels, logp_t=logp_t)


def dpo_head_forward_shared(dims, W, batch, y_ft_list, ref_logp, beta):
    """DPO head when a pair is stored once as prompt | chosen response | rejected response (the
    prompt rows are shared).  The first token of either response is predicted by the LAST PROMPT
    row, the others by the response rows before them; everything else is dpo_head_forward.
    Sequence numbering of logp / ref_logp stays 2i = chosen, 2i+1 = rejected."""
    seg = np.asarray(batch.seg_offsets, dtype=np.int64)
    base = len(batch.prefill_lens) + len(batch.decode_ctx)
    logp, saved = [], []
    for i, y_seq in enumerate(y_ft_list):
        y_seq = np.asarray(y_seq, F64)
        ids = np.asarray(batch.token_ids[seg[base + i]:seg[base + i + 1]])
        P, Rc = int(batch.ft_prompt_lens[i]), int(batch.ft_chosen_lens[i])
        L = y_seq.shape[0]
        Rr = L - P - Rc
        for start, R in ((P, Rc), (P + Rc, Rr)):
            rows = np.concatenate([[P - 1], np.arange(start, start + R - 1)])
            lp, sv = rows_logprob(dims, W, y_seq, rows, ids[start:start + R])
            sv["y"], sv["pair"] = y_seq, i
            logp.append(lp)
            saved.append(sv)
    logp = np.array(logp, F64)
    loss, loss_mean, clpd, win, z, dlogp = dpo_pair_loss(logp, ref_logp, beta)
    return dict(logp=logp, loss_per_pair=loss, loss_mean=loss_mean, clpd=clpd, win=win, z=z, dlogp=dlogp, saved=saved)


def dpo_head_backward_shared(dims, W, head, n_pairs):
    """dpo_head_backward for the shared-prompt layout: the two sequences of a pair scatter into the
    rows of one stored pair, and the last prompt row receives the gradient of both."""
    dys_seq, dE, dgf = dpo_head_backward(dims, W, head)
    return [dys_seq[2 * i] + dys_seq[2 * i + 1] for i in range(n_pairs)], dE, dgf


def dpo_head_backward(dims, W, head):
    """dlogits_t = dlogp_s * (onehot(label_t) - softmax(logits_t)) ; dn = dlogits E ;
    dE += dlogits^T n ; final RMSNorm backward.  Returns dL/dy per ft sequence (zero on rows that
    carry no loss), dE (head contribution only) and dgf."""
    E = _w(W, "E")
    dE = np.zeros_like(E)
    dgf = np.zeros(E.shape[1], F64)
    dys = []
    for s, sv in enumerate(head["saved"]):
        p = np.exp(sv["logits"] - sv["lse"][:, None])
        dl = -p
        dl[np.arange(len(sv["rows"])), sv["labels"]] += 1.0
        dl *= head["dlogp"][s]
        dn = dl @ E
        dE += dl.T @ sv["n"]
        dyr, dg = rmsnorm_bwd(dn, sv["y"][sv["rows"]], _w(W, "gf"), sv["rf"])
        dgf += dg
        dy = np.zeros_like(sv["y"])
        dy[sv["rows"]] = dyr
        dys.append(dy)
    return dys, dE, dgf


def layer_backward_lora(dims, W, lora, saved, dy_list):
    """Backward of the layer over the fine-tune sequences when only the adapter is trained: the
    base weights and gains are frozen, so the pass produces dx per sequence and the summed
    gradients of a_p, b_p for p in q, k, v, o - no base-weight gradient is formed."""
    grads = {}
    for p in ("q", "k", "v", "o"):
        grads["a_" + p] = np.zeros_like(np.asarray(lora["a_" + p], F64))
        grads["b_" + p] = np.zeros_like(np.asarray(lora["b_" + p], F64))

    def acc(p, dA, dB):
        grads["a_" + p] += dA
        grads["b_" + p] += dB

    dxs = []
    for sv, dy in zip(saved, dy_list):
        dy = np.asarray(dy, F64)
        L = dy.shape[0]
        dHm = dy @ _w(W, "wd")
        dx1 = dy.copy()
        sg = sigmoid(sv["G"])
        dU = dHm * (sv["G"] * sg)
        dG = dHm * sv["U"] * sg * (1.0 + sv["G"] * (1.0 - sg))
        db = dG @ _w(W, "wg") + dU @ _w(W, "wu")
        dxa, _ = rmsnorm_bwd(db, sv["x1"], _w(W, "g2"), sv["r2"])
        dx1 += dxa
        attn = sv["o"].reshape(L, -1)
        dattn, dA, dB = adapted_linear_bwd(dx1, attn, _w(W, "wo"), lora, "o")
        acc("o", dA, dB)
        dx = dx1.copy()
        dq, dk, dv = causal_attention_bwd(dattn.reshape(sv["o"].shape), sv["q"], sv["k"], sv["v"], sv["o"], sv["P"])
        dq = rope(dq, sv["pos"], dims.rope_theta, sign=-1.0)
        dk = rope(dk, sv["pos"], dims.rope_theta, sign=-1.0)
        da = np.zeros_like(sv["a"])
        for p, g, wn in (("q", dq.reshape(L, -1), "wq"), ("k", dk.reshape(L, -1), "wk"), ("v", dv.reshape(L, -1), "wv")):
            du, dA, dB = adapted_linear_bwd(g, sv["a"], _w(W, wn), lora, p)
            da += du
            acc(p, dA, dB)
        dxa, _ = rmsnorm_bwd(da, sv["x"], _w(W, "g1"), sv["r1"])
        dx += dxa
        dxs.append(dx)
    return dxs, grads


# --------------------------------------------------------------------------- cache-pruning statistics

def rolling_mean_update(abar, norms, t_count):
    """Running mean of the head norms (Section 4.3): after the update abar is the mean of the
    t_count norms seen so far, abar <- abar + (norm - abar) / t_count.  abar, norms [n, H];
    t_count [n] = number of decode iterations of each request including this one."""
    abar, norms = np.asarray(abar, F64), np.asarray(norms, F64)
    return abar + (norms - abar) / np.asarray(t_count, F64)[:, None]


def head_budget(abar, c_total):
    """Per-head cache capacity (Section 4.3): w_h = abar_h / sum_j abar_j, C_h = floor(w_h C_total),
    and the capacity the floors leave over goes, one unit each, to the heads with the largest
    weights (ties: the lower head index first).  Returns int64 [H] with sum == c_total."""
    abar = np.asarray(abar, F64)
    w = abar / np.sum(abar)
    c = np.floor(w * F64(c_total)).astype(np.int64)
    left = int(c_total) - int(c.sum())
    order = sorted(range(len(w)), key=lambda h: (-w[h], h))
    for h in order[:left]:
        c[h] += 1
    return c


def prune_flags(norms, t_now, t_last_used, window, tau):
    """Prune predicate of Section 4.3 per (request, head): t - t_last_used > W  or  norm < tau.
    Reading: t_last_used is the last iteration at which that head's norm reached tau; it is
    returned updated (t_now where norm >= tau).  t_now [n], t_last_used [n, H] integers."""
    norms = np.asarray(norms, F64)
    t_now = np.asarray(t_now, np.int64)[:, None]
    last = np.asarray(t_last_used, np.int64)
    low = norms < tau
    flags = ((t_now - last) > window) | low
    return flags, np.where(low, last, t_now)


# --------------------------------------------------------------------------- closing the loop

def next_token_logits(dims, W, y_rows):
    """Logits of the token that follows each given row (the decode rows, or the last row of a
    prefill request): final RMSNorm, tied head E.  Returns logits [n, V] and the greedy choice
    argmax (lowest index on ties) - what the serving loop samples from and checks for
    end-of-sequence (Section 4.2, CheckEnd)."""
    n, _ = rmsnorm(np.asarray(y_rows, F64), _w(W, "gf"), dims.rms_eps)
    logits = n @ _w(W, "E").T
    return logits, np.argmax(logits, axis=1)


def adamw_step(param, grad, m, v, step, lr, beta1, beta2, eps, weight_decay):
    """One AdamW update (decoupled weight decay), the optimizer step that turns the gradients of an
    iteration into the model the next iteration sees (Section 2.1: later requests benefit from the
    updated model).  step counts from 1.
      m <- b1 m + (1-b1) g ; v <- b2 v + (1-b2) g^2 ; mhat = m/(1-b1^t) ; vhat = v/(1-b2^t)
      p <- p - lr * (mhat / (sqrt(vhat) + eps) + wd * p)
    Returns the new (param, m, v)."""
    p, g = np.asarray(param, F64), np.asarray(grad, F64)
    m = beta1 * np.asarray(m, F64) + (1.0 - beta1) * g
    v = beta2 * np.asarray(v, F64) + (1.0 - beta2) * g * g
    mhat = m / (1.0 - beta1 ** step)
    vhat = v / (1.0 - beta2 ** step)
    p = p - lr * (mhat / (np.sqrt(vhat) + eps) + weight_decay * p)
    return p, m, v


# --------------------------------------------------------------------------- whole iteration

def hybrid_iteration(dims, W, batch, x, cache_k, cache_v, ref_logp, beta, backward=True, lora=None, extras=None):
    """Forward of all rows, DPO head over the ft sequences, and the backward pass of the ft
    sequences.  Returns a dict with y, slots, the head outputs, and the gradients (with `lora`:
    the adapter gradients only, the base model being frozen)."""
    y, slots, saved = layer_forward(dims, W, batch, x, cache_k, cache_v, lora, extras)
    seg = np.asarray(batch.seg_offsets, dtype=np.int64)
    base = len(batch.prefill_lens) + len(batch.decode_ctx)
    y_ft = [y[seg[base + s]:seg[base + s + 1]] for s in range(len(batch.ft_lens))]
    shared = getattr(batch, "ft_chosen_lens", None) is not None
    head = (dpo_head_forward_shared if shared else dpo_head_forward)(dims, W, batch, y_ft, ref_logp, beta)
    out = dict(y=y, slots=slots, head=head, saved=saved)
    if backward:
        dys, dE, dgf = dpo_head_backward_shared(dims, W, head, len(y_ft)) if shared else dpo_head_backward(dims, W, head)
        if lora is not None:
            dxs, grads = layer_backward_lora(dims, W, lora, saved, dys)
        else:
            dxs, grads = layer_backward(dims, W, saved, dys)
            grads["E"] = dE
            grads["gf"] = dgf
        out.update(dy_ft=np.concatenate(dys), dx_ft=np.concatenate(dxs), grads=grads)
    return out


def new_cache(num_blocks, n_kv_heads, block_size, head_dim):
    return np.zeros((num_blocks, n_kv_heads, block_size, head_dim), F64)


def load_context(cache, block_tables, block_size, ctx_rows):
    """Place each decode request's already-cached rows [ctx, Hkv, hd] at its block-table slots."""
    for j, rows in enumerate(ctx_rows):
        if len(rows):
            kv_append(cache, np.asarray(rows, F64), slot_mapping(block_tables[j], block_size, 0, len(rows)))
