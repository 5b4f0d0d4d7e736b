"""ctypes binding of libmace_hip.so: the same entry points as include/mace.h, argument
marshalling only.  Device buffers are torch tensors (torch is used for memory and streams);
every step of the path runs inside the library's HIP kernels.  There is no fallback: if the
library is missing or a call fails, an exception is raised."""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import torch

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libmace_hip.so")
_lib = None

MACE_F32, MACE_BF16 = 0, 1

EXPORTS = [
    "mace_create", "mace_destroy", "mace_last_error", "mace_fwd_saved_bytes", "mace_workspace_bytes",
    "mace_kv_slot_mapping", "mace_kv_cache_append", "mace_kv_cache_gather", "mace_hybrid_layer_fwd",
    "mace_hybrid_layer_bwd", "mace_hybrid_layer_fwd_lora", "mace_hybrid_layer_bwd_lora", "mace_dpo_logprob_loss", "mace_dpo_logprob_loss_shared",
    "mace_next_token_logits", "mace_adamw_step", "mace_head_norm_stats", "mace_kv_head_budget", "mace_profile_enable", "mace_profile_collect",
    "mace_set_option", "mace_launch_plan", "mace_next_token_logits_static", "mace_gemm_bf16",
]
MACE_OPT_HEAD_TWO_PASS, MACE_OPT_SINGLE_STREAM, MACE_OPT_DECODE_CHUNK = 1, 2, 3


class MaceError(RuntimeError):
    pass


class ModelT(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32), ("head_dim", C.c_int32),
                ("d_ff", C.c_int32), ("vocab", C.c_int32), ("rms_eps", C.c_float), ("rope_theta", C.c_float),
                ("io_dtype", C.c_int32)]


class LayerWT(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g_attn", "wq", "wk", "wv", "wo", "g_mlp", "w_gate", "w_up", "w_down")]


class LayerGradsT(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("g_attn", "wq", "wk", "wv", "wo", "g_mlp", "w_gate", "w_up", "w_down")]


_LORA_NAMES = ("a_q", "b_q", "a_k", "b_k", "a_v", "b_v", "a_o", "b_o")


class LoraT(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LORA_NAMES] + [("rank", C.c_int32), ("scale", C.c_float)]


class LoraGradsT(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _LORA_NAMES]


class KvCacheT(C.Structure):
    _fields_ = [("k", C.c_void_p), ("v", C.c_void_p), ("num_blocks", C.c_int64), ("block_size", C.c_int32)]


class BatchT(C.Structure):
    _fields_ = [("n_prefill", C.c_int32), ("n_decode", C.c_int32), ("n_ft_seq", C.c_int32), ("n_tokens", C.c_int32),
                ("seg_offsets_host", C.c_void_p), ("seg_offsets", C.c_void_p), ("positions", C.c_void_p),
                ("slot_mapping", C.c_void_p), ("block_tables", C.c_void_p), ("context_lens_host", C.c_void_p),
                ("context_lens", C.c_void_p), ("max_blocks_per_req", C.c_int32), ("prefill_block_tables", C.c_void_p),
                ("prefill_prefix_lens_host", C.c_void_p), ("prefill_prefix_lens", C.c_void_p), ("max_blocks_per_prefill", C.c_int32),
                ("ft_excl_lo", C.c_void_p), ("ft_excl_hi", C.c_void_p), ("decode_head_norms", C.c_void_p)]


class GemmPlanT(C.Structure):
    _fields_ = [("name", C.c_char * 32), ("layout", C.c_int32), ("tile_m", C.c_int32), ("tile_n", C.c_int32), ("k_splits", C.c_int32),
                ("on_side_stream", C.c_int32), ("m", C.c_int64), ("n", C.c_int64), ("k", C.c_int64)]


class GemmDescT(C.Structure):
    _fields_ = [("layout_a", C.c_int32), ("layout_b", C.c_int32), ("M", C.c_int32), ("N", C.c_int32), ("K", C.c_int32),
                ("lda", C.c_int64), ("ldb", C.c_int64), ("ldc", C.c_int64), ("ldr", C.c_int64),
                ("a", C.c_void_p), ("a_lo", C.c_void_p), ("b", C.c_void_p), ("b_up", C.c_void_p),
                ("c", C.c_void_p), ("c_lo", C.c_void_p), ("c_gu", C.c_void_p), ("resid", C.c_void_p),
                ("out_bf16", C.c_int32), ("resid_kind", C.c_int32), ("swiglu", C.c_int32), ("kernel", C.c_int32),
                ("rope_cs", C.c_void_p), ("rope_rotate", C.c_int32)]


class ProfileEntryT(C.Structure):
    _fields_ = [("name", C.c_char * 48), ("launches", C.c_int64), ("side_launches", C.c_int64), ("ms", C.c_double), ("flops", C.c_double),
                ("bytes", C.c_double)]


def lib_path() -> str:
    return _LIB_PATH


def load():
    """Load the HIP library (built in-tree by paper_2510_03283_amd.build); fail loudly if absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise MaceError(f"{_LIB_PATH} is missing: build it with `python -m paper_2510_03283_amd.build`")
    lib = C.CDLL(_LIB_PATH)
    vp, i32, i64, sz, f32 = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t, C.c_float
    lib.mace_create.argtypes = [C.POINTER(vp), C.POINTER(ModelT)]
    lib.mace_create.restype = C.c_int
    lib.mace_destroy.argtypes = [vp]
    lib.mace_destroy.restype = None
    lib.mace_last_error.argtypes = []
    lib.mace_last_error.restype = C.c_char_p
    lib.mace_fwd_saved_bytes.argtypes = [vp, i32]
    lib.mace_fwd_saved_bytes.restype = sz
    lib.mace_workspace_bytes.argtypes = [vp, i32, i32, i32, i32, i32]
    lib.mace_workspace_bytes.restype = sz
    lib.mace_kv_slot_mapping.argtypes = [vp, i32, i32, i32, i32, vp]
    lib.mace_kv_slot_mapping.restype = C.c_int
    lib.mace_kv_cache_append.argtypes = [vp, C.POINTER(KvCacheT), vp, vp, vp, i32, vp]
    lib.mace_kv_cache_append.restype = C.c_int
    lib.mace_kv_cache_gather.argtypes = [vp, C.POINTER(KvCacheT), vp, i32, vp, vp, vp, vp]
    lib.mace_kv_cache_gather.restype = C.c_int
    lib.mace_hybrid_layer_fwd.argtypes = [vp, C.POINTER(LayerWT), C.POINTER(BatchT), C.POINTER(KvCacheT), vp, vp, vp, vp, sz, vp]
    lib.mace_hybrid_layer_fwd.restype = C.c_int
    lib.mace_hybrid_layer_bwd.argtypes = [vp, C.POINTER(LayerWT), C.POINTER(BatchT), vp, vp, vp, vp, C.POINTER(LayerGradsT), C.c_int, vp, sz, vp]
    lib.mace_hybrid_layer_bwd.restype = C.c_int
    lib.mace_hybrid_layer_fwd_lora.argtypes = [vp, C.POINTER(LayerWT), C.POINTER(LoraT), C.POINTER(BatchT), C.POINTER(KvCacheT), vp, vp, vp, vp, sz, vp]
    lib.mace_hybrid_layer_fwd_lora.restype = C.c_int
    lib.mace_hybrid_layer_bwd_lora.argtypes = [vp, C.POINTER(LayerWT), C.POINTER(LoraT), C.POINTER(BatchT), vp, vp, vp, vp, C.POINTER(LoraGradsT), C.c_int, vp, sz, vp]
    lib.mace_hybrid_layer_bwd_lora.restype = C.c_int
    lib.mace_dpo_logprob_loss.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, f32, vp, vp, vp, vp, vp, vp, vp, vp, C.c_int, vp, sz, vp]
    lib.mace_dpo_logprob_loss.restype = C.c_int
    lib.mace_next_token_logits.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp, sz, vp]
    lib.mace_next_token_logits.restype = C.c_int
    lib.mace_next_token_logits_static.argtypes = [vp, vp, vp, i32, vp, vp, vp, vp, vp]
    lib.mace_next_token_logits_static.restype = C.c_int
    lib.mace_adamw_step.argtypes = [vp, vp, vp, vp, vp, vp, i64, f32, f32, f32, f32, f32, i32, vp]
    lib.mace_adamw_step.restype = C.c_int
    lib.mace_head_norm_stats.argtypes = [vp, vp, vp, i32, i32, vp, vp, i32, f32, vp, vp]
    lib.mace_head_norm_stats.restype = C.c_int
    lib.mace_kv_head_budget.argtypes = [vp, i32, i64, vp]
    lib.mace_kv_head_budget.restype = C.c_int
    lib.mace_dpo_logprob_loss_shared.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, i32, vp, f32, vp, vp, vp, vp, vp, vp, vp, vp, C.c_int, vp, sz, vp]
    lib.mace_dpo_logprob_loss_shared.restype = C.c_int
    lib.mace_profile_enable.argtypes = [vp, C.c_int]
    lib.mace_profile_enable.restype = C.c_int
    lib.mace_profile_collect.argtypes = [vp, C.POINTER(ProfileEntryT), i32, C.POINTER(i32)]
    lib.mace_profile_collect.restype = C.c_int
    lib.mace_set_option.argtypes = [vp, i32, i32]
    lib.mace_set_option.restype = C.c_int
    lib.mace_launch_plan.argtypes = [vp, C.POINTER(GemmPlanT), i32, C.POINTER(i32)]
    lib.mace_launch_plan.restype = C.c_int
    lib.mace_gemm_bf16.argtypes = [vp, C.POINTER(GemmDescT), vp]
    lib.mace_gemm_bf16.restype = C.c_int
    _lib = lib
    return lib


def _check(rc: int, what: str):
    if rc != 0:
        raise MaceError(f"{what} failed ({rc}): {load().mace_last_error().decode()}")


def _dev(t: Optional[torch.Tensor]):
    if t is None:
        return None
    assert t.is_cuda and t.is_contiguous(), "device tensors must be contiguous GPU tensors"
    return C.c_void_p(t.data_ptr())


def _host_i32(t):
    """Host int32 array -> (keep-alive numpy array, pointer)."""
    import numpy as np
    a = np.ascontiguousarray(t, dtype=np.int32)
    return a, C.c_void_p(a.ctypes.data)


def _stream(stream=None):
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


def mace_create(d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab, rms_eps, rope_theta, io_dtype):
    h = C.c_void_p()
    m = ModelT(d_model, n_q_heads, n_kv_heads, head_dim, d_ff, vocab, rms_eps, rope_theta, io_dtype)
    _check(load().mace_create(C.byref(h), C.byref(m)), "mace_create")
    return h


def mace_destroy(h):
    load().mace_destroy(h)


def mace_set_option(h, option: int, value: int):
    _check(load().mace_set_option(h, int(option), int(value)), "mace_set_option")


def mace_launch_plan(h) -> list:
    """GEMM launch decisions of the last iteration call on this handle, in launch order."""
    arr = (GemmPlanT * 256)()
    n = C.c_int32(0)
    _check(load().mace_launch_plan(h, arr, 256, C.byref(n)), "mace_launch_plan")
    return [dict(name=arr[i].name.decode(), layout=int(arr[i].layout), tile=(int(arr[i].tile_m), int(arr[i].tile_n)),
                 k_splits=int(arr[i].k_splits), on_side_stream=int(arr[i].on_side_stream), m=int(arr[i].m), n=int(arr[i].n),
                 k=int(arr[i].k)) for i in range(min(n.value, 256))]


def mace_gemm_bf16(h, layout_a: int, layout_b: int, M: int, N: int, K: int, a, b, c, a_lo=None, resid=None, b_up=None, c_lo=None,
                   c_gu=None, lda=None, ldb=None, ldc=None, ldr=None, swiglu=False, kernel=0, rope_cs=None, rope_rotate=True, stream=None):
    """The dense contraction kernel on its own (argument marshalling only; see include/mace.h)."""
    d = GemmDescT()
    d.layout_a, d.layout_b, d.M, d.N, d.K = layout_a, layout_b, M, N, K
    d.lda = lda if lda is not None else (K if layout_a == 0 else M)
    d.ldb = ldb if ldb is not None else (K if layout_b == 0 else N)
    d.ldc = ldc if ldc is not None else N
    d.ldr = ldr if ldr is not None else d.ldc
    d.a, d.a_lo, d.b, d.b_up = _dev(a), _dev(a_lo), _dev(b), _dev(b_up)
    d.c, d.c_lo, d.c_gu, d.resid = _dev(c), _dev(c_lo), _dev(c_gu), _dev(resid)
    d.out_bf16 = 1 if c.dtype == torch.bfloat16 else 0
    d.resid_kind = 0 if resid is None else (2 if resid.dtype == torch.bfloat16 else 1)
    d.swiglu, d.kernel = int(swiglu), int(kernel)
    d.rope_cs, d.rope_rotate = _dev(rope_cs), int(bool(rope_rotate))
    _check(load().mace_gemm_bf16(h, C.byref(d), _stream(stream)), "mace_gemm_bf16")


def mace_fwd_saved_bytes(h, n_ft_tokens: int) -> int:
    return int(load().mace_fwd_saved_bytes(h, n_ft_tokens))


def mace_workspace_bytes(h, n_tokens, n_ft_tokens, n_decode, max_context, n_loss_rows) -> int:
    return int(load().mace_workspace_bytes(h, n_tokens, n_ft_tokens, n_decode, max_context, n_loss_rows))


def mace_kv_slot_mapping(block_table, block_size: int, start_pos: int, n: int):
    """Host-side slot computation; returns a numpy int32 array."""
    import numpy as np
    bt, btp = _host_i32(block_table)
    out = np.empty(n, dtype=np.int32)
    _check(load().mace_kv_slot_mapping(btp, len(bt), block_size, start_pos, n, C.c_void_p(out.ctypes.data)), "mace_kv_slot_mapping")
    return out


def kv_cache_struct(k: torch.Tensor, v: torch.Tensor, num_blocks: int, block_size: int) -> KvCacheT:
    return KvCacheT(k.data_ptr(), v.data_ptr(), num_blocks, block_size)


def mace_kv_cache_append(h, cache: KvCacheT, k_new, v_new, slot_mapping, n: int, stream=None):
    _check(load().mace_kv_cache_append(h, C.byref(cache), _dev(k_new), _dev(v_new), _dev(slot_mapping), n, _stream(stream)), "mace_kv_cache_append")


def mace_kv_cache_gather(h, cache: KvCacheT, block_table, ctx_len: int, k_out, v_out, slots_out=None, stream=None):
    _check(load().mace_kv_cache_gather(h, C.byref(cache), _dev(block_table), ctx_len, _dev(k_out), _dev(v_out), _dev(slots_out), _stream(stream)), "mace_kv_cache_gather")


def layer_weights_struct(w: dict) -> LayerWT:
    """w: dict of device tensors keyed g1, wq, wk, wv, wo, g2, wg, wu, wd."""
    return LayerWT(*[w[k].data_ptr() for k in ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")])


def layer_grads_struct(g: dict) -> LayerGradsT:
    return LayerGradsT(*[(g[k].data_ptr() if g.get(k) is not None else None) for k in ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")])


class BatchDesc:
    """Owns the host arrays a mace_batch_t points to, next to the struct itself."""

    def __init__(self, n_prefill, n_decode, n_ft_seq, n_tokens, seg_offsets_host, seg_offsets, positions,
                 slot_mapping, block_tables, context_lens_host, context_lens, max_blocks_per_req, decode_head_norms=None,
                 prefill_block_tables=None, prefill_prefix_lens_host=None, prefill_prefix_lens=None, max_blocks_per_prefill=0,
                 ft_excl_lo=None, ft_excl_hi=None):
        self._seg, segp = _host_i32(seg_offsets_host)
        self._ctx, ctxp = _host_i32(context_lens_host)
        self._keep = (seg_offsets, positions, slot_mapping, block_tables, context_lens, decode_head_norms,
                      prefill_block_tables, prefill_prefix_lens, ft_excl_lo, ft_excl_hi)
        pfxp = None
        if prefill_prefix_lens_host is not None:
            self._pfx, pfxp = _host_i32(prefill_prefix_lens_host)
        self.struct = BatchT(n_prefill, n_decode, n_ft_seq, n_tokens, segp, _dev(seg_offsets), _dev(positions),
                             _dev(slot_mapping), _dev(block_tables), ctxp if n_decode else None,
                             _dev(context_lens), max_blocks_per_req, _dev(prefill_block_tables), pfxp,
                             _dev(prefill_prefix_lens), max_blocks_per_prefill, _dev(ft_excl_lo), _dev(ft_excl_hi),
                             _dev(decode_head_norms))


def mace_hybrid_layer_fwd(h, w: LayerWT, batch: BatchDesc, cache: Optional[KvCacheT], x, y, saved, workspace, stream=None):
    _check(load().mace_hybrid_layer_fwd(h, C.byref(w), C.byref(batch.struct), C.byref(cache) if cache is not None else None,
                                        _dev(x), _dev(y), _dev(saved), _dev(workspace), workspace.numel() * workspace.element_size(),
                                        _stream(stream)), "mace_hybrid_layer_fwd")


def mace_hybrid_layer_bwd(h, w: LayerWT, batch: BatchDesc, x, dy_ft, saved, dx_ft, grads: LayerGradsT, accumulate, workspace, stream=None):
    _check(load().mace_hybrid_layer_bwd(h, C.byref(w), C.byref(batch.struct), _dev(x), _dev(dy_ft), _dev(saved), _dev(dx_ft),
                                        C.byref(grads), int(accumulate), _dev(workspace), workspace.numel() * workspace.element_size(),
                                        _stream(stream)), "mace_hybrid_layer_bwd")


def lora_struct(l: dict, rank: int, scale: float) -> LoraT:
    """l: dict of device tensors keyed a_q, b_q, ..., b_o (io dtype)."""
    return LoraT(*[l[k].data_ptr() for k in _LORA_NAMES], int(rank), float(scale))


def lora_grads_struct(g: dict) -> LoraGradsT:
    return LoraGradsT(*[(g[k].data_ptr() if g.get(k) is not None else None) for k in _LORA_NAMES])


def mace_hybrid_layer_fwd_lora(h, w: LayerWT, lora: LoraT, batch: BatchDesc, cache: Optional[KvCacheT], x, y, saved, workspace, stream=None):
    _check(load().mace_hybrid_layer_fwd_lora(h, C.byref(w), C.byref(lora), C.byref(batch.struct),
                                             C.byref(cache) if cache is not None else None, _dev(x), _dev(y), _dev(saved),
                                             _dev(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "mace_hybrid_layer_fwd_lora")


def mace_hybrid_layer_bwd_lora(h, w: LayerWT, lora: LoraT, batch: BatchDesc, x, dy_ft, saved, dx_ft, grads: LoraGradsT, accumulate,
                               workspace, stream=None):
    _check(load().mace_hybrid_layer_bwd_lora(h, C.byref(w), C.byref(lora), C.byref(batch.struct), _dev(x), _dev(dy_ft), _dev(saved),
                                             _dev(dx_ft), C.byref(grads), int(accumulate), _dev(workspace),
                                             workspace.numel() * workspace.element_size(), _stream(stream)),
           "mace_hybrid_layer_bwd_lora")


def mace_dpo_logprob_loss(h, h_ft, g_final, w_lm, token_ids, ft_seq_offsets, ft_seq_offsets_host, prompt_lens, prompt_lens_host,
                          n_pairs, ref_logp, beta, logp_out, loss_per_pair, loss_mean, clpd_out, win_out, dh_ft, dw_lm, dg_final,
                          accumulate, workspace, stream=None):
    so, sop = _host_i32(ft_seq_offsets_host)
    pl, plp = _host_i32(prompt_lens_host)
    _check(load().mace_dpo_logprob_loss(h, _dev(h_ft), _dev(g_final), _dev(w_lm), _dev(token_ids), _dev(ft_seq_offsets), sop,
                                        _dev(prompt_lens), plp, n_pairs, _dev(ref_logp), float(beta), _dev(logp_out),
                                        _dev(loss_per_pair), _dev(loss_mean), _dev(clpd_out), _dev(win_out), _dev(dh_ft),
                                        _dev(dw_lm), _dev(dg_final), int(accumulate), _dev(workspace),
                                        workspace.numel() * workspace.element_size(), _stream(stream)), "mace_dpo_logprob_loss")


def mace_dpo_logprob_loss_shared(h, h_ft, g_final, w_lm, token_ids, pair_offsets, pair_offsets_host, prompt_lens, prompt_lens_host,
                                 chosen_lens, chosen_lens_host, n_pairs, ref_logp, beta, logp_out, loss_per_pair, loss_mean, clpd_out,
                                 win_out, dh_ft, dw_lm, dg_final, accumulate, workspace, stream=None):
    so, sop = _host_i32(pair_offsets_host)
    pl, plp = _host_i32(prompt_lens_host)
    cl, clp = _host_i32(chosen_lens_host)
    _check(load().mace_dpo_logprob_loss_shared(h, _dev(h_ft), _dev(g_final), _dev(w_lm), _dev(token_ids), _dev(pair_offsets), sop,
                                               _dev(prompt_lens), plp, _dev(chosen_lens), clp, n_pairs, _dev(ref_logp), float(beta),
                                               _dev(logp_out), _dev(loss_per_pair), _dev(loss_mean), _dev(clpd_out), _dev(win_out),
                                               _dev(dh_ft), _dev(dw_lm), _dev(dg_final), int(accumulate), _dev(workspace),
                                               workspace.numel() * workspace.element_size(), _stream(stream)),
           "mace_dpo_logprob_loss_shared")


def mace_next_token_logits(h, y, row_idx, n, g_final, w_lm, logits_out, next_token, workspace, stream=None):
    _check(load().mace_next_token_logits(h, _dev(y), _dev(row_idx), int(n), _dev(g_final), _dev(w_lm), _dev(logits_out), _dev(next_token),
                                         _dev(workspace), workspace.numel() * workspace.element_size(), _stream(stream)),
           "mace_next_token_logits")


def mace_next_token_logits_static(h, y, row_idx, n, g_final, w_lm, logits_out, next_token, stream=None):
    _check(load().mace_next_token_logits_static(h, _dev(y), _dev(row_idx), int(n), _dev(g_final), _dev(w_lm), _dev(logits_out),
                                                _dev(next_token), _stream(stream)), "mace_next_token_logits_static")


def mace_adamw_step(h, param, master, grad, m, v, lr, beta1, beta2, eps, weight_decay, step, stream=None):
    _check(load().mace_adamw_step(h, _dev(param), _dev(master), _dev(grad), _dev(m), _dev(v), param.numel(), float(lr), float(beta1),
                                  float(beta2), float(eps), float(weight_decay), int(step), _stream(stream)), "mace_adamw_step")


def mace_head_norm_stats(h, norms, t_count, abar, last_used=None, window=0, tau=0.0, prune=None, stream=None):
    n, H = norms.shape
    _check(load().mace_head_norm_stats(h, _dev(norms), _dev(t_count), n, H, _dev(abar), _dev(last_used), int(window), float(tau),
                                       _dev(prune), _stream(stream)), "mace_head_norm_stats")


def mace_kv_head_budget(abar, c_total: int):
    """Host-side capacity split; abar: sequence of positive floats.  Returns a numpy int64 array."""
    import numpy as np
    a = np.ascontiguousarray(abar, dtype=np.float64)
    out = np.empty(len(a), dtype=np.int64)
    _check(load().mace_kv_head_budget(C.c_void_p(a.ctypes.data), len(a), int(c_total), C.c_void_p(out.ctypes.data)), "mace_kv_head_budget")
    return out


PROFILE_CLASSES = ["gemm_nt", "gemm_nn", "gemm_tn", "attn_fwd_prefill", "attn_fwd_ft", "attn_decode", "attn_bwd",
                   "rmsnorm", "rope", "swiglu", "logsoftmax", "dlogits", "misc"]


def mace_profile_enable(h, on):
    """on: False/0 off, True/1 all kernel classes, or a list of class names to time only those."""
    if isinstance(on, (list, tuple, set)):
        mask = 0
        for name in on:
            mask |= 1 << (PROFILE_CLASSES.index(name) + 1)
        on = mask
    _check(load().mace_profile_enable(h, int(on)), "mace_profile_enable")


def mace_profile_collect(h) -> dict:
    """Per kernel class: launches, summed ms, summed algorithmic flops and bytes."""
    arr = (ProfileEntryT * 16)()
    n = C.c_int32(0)
    _check(load().mace_profile_collect(h, arr, 16, C.byref(n)), "mace_profile_collect")
    return {arr[i].name.decode(): dict(launches=int(arr[i].launches), side_launches=int(arr[i].side_launches), ms=float(arr[i].ms), flops=float(arr[i].flops),
                                       bytes=float(arr[i].bytes)) for i in range(n.value)}
