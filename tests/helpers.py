"""Shared test helpers: run the CPU oracle on a synthetic workload, error metrics."""
import numpy as np

from oracle import mace_oracle as O


def run_oracle(wl, backward=True, lora=None):
    m, b = wl.dims, wl.batch
    ck = O.new_cache(b.num_blocks, m.n_kv_heads, b.block_size, m.head_dim)
    cv = O.new_cache(b.num_blocks, m.n_kv_heads, b.block_size, m.head_dim)
    if len(b.decode_ctx) and wl.ctx_k is not None:
        O.load_context(ck, b.decode_block_tables, b.block_size, wl.ctx_k)
        O.load_context(cv, b.decode_block_tables, b.block_size, wl.ctx_v)
    if getattr(wl, "pre_k", None) is not None:
        O.load_context(ck, b.prefill_block_tables, b.block_size, wl.pre_k)
        O.load_context(cv, b.prefill_block_tables, b.block_size, wl.pre_v)
    extras = {}
    if len(b.ft_lens) == 0:       # inference-only batch: there is no DPO head to run
        y, slots, saved = O.layer_forward(m, wl.weights, b, wl.x, ck, cv, lora, extras)
        out = dict(y=y, slots=slots, saved=saved)
    else:
        out = O.hybrid_iteration(m, wl.weights, b, wl.x, ck, cv, wl.ref_logp, wl.beta, backward=backward, lora=lora, extras=extras)
    out["head_norms"] = extras["head_norms"]
    out["cache_k"], out["cache_v"] = ck, cv
    return out


def max_abs_norm_err(a, b):
    """max|a-b| / max|b| (b = oracle)."""
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.max(np.abs(a - b)) / max(np.max(np.abs(b)), 1e-300))


def rel_fro_err(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))
