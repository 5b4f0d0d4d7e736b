"""Runs one hybrid iteration of a synthetic workload on the GPU through the C-ABI binding.

Only plumbing lives here: uploading the seeded inputs, allocating buffers with torch, and
calling the library entry points in order (forward of all rows, DPO head, backward of the
fine-tune rows).  Used by the GPU tests, the smoke check and bench.py."""
from __future__ import annotations

import numpy as np
import torch

from . import binding as B
from .synth import Workload

_WNAMES = ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")


class DeviceIteration:
    def __init__(self, wl: Workload, device: str = "cuda:0", load_cache: bool = True, device_cache_seed=None, lora=None,
                 options=None):
        """options: {binding.MACE_OPT_*: value} set on the handle right after it is created.
        lora: adapter dict of synth.make_lora - the iteration then runs the adapter variant (base
        model frozen, adapter gradients only).
        device_cache_seed: fill the cached contexts with N(0,1) values drawn on the GPU (torch
        generator) instead of uploading wl.ctx_k / ctx_v - for benchmark workloads whose cache
        (tens of GB) is too large to generate on the host.  Not used by parity tests."""
        self.wl = wl
        self.dev = torch.device(device)
        m, b = wl.dims, wl.batch
        self.io_dtype = torch.bfloat16 if m.io_bf16 else torch.float32
        self.h = B.mace_create(m.d_model, m.n_q_heads, m.n_kv_heads, m.head_dim, m.d_ff, m.vocab, m.rms_eps,
                               m.rope_theta, B.MACE_BF16 if m.io_bf16 else B.MACE_F32)
        for opt, val in (options or {}).items():
            B.mace_set_option(self.h, opt, val)
        up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(self.dev)
        upio = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(self.dev).to(self.io_dtype).contiguous()
        self.w = {k: upio(wl.weights[k]) for k in _WNAMES}
        self.E = upio(wl.weights["E"])
        self.gf = upio(wl.weights["gf"])
        self.w_struct = B.layer_weights_struct(self.w)
        self.x = upio(wl.x)
        self.lora = None
        if lora is not None:
            self.lora_dev = {k: upio(lora[k]) for k in B._LORA_NAMES}
            self.lora = B.lora_struct(self.lora_dev, lora["rank"], lora["scale"])

        # descriptor arrays
        self.T, self.Tp, self.Td, self.Tf = b.n_tokens, b.t_prefill, b.t_decode, b.t_ft
        self.Ti = self.Tp + self.Td
        self.R = b.n_loss_rows
        seg = np.asarray(b.seg_offsets, dtype=np.int32)
        slots = []
        pfx = b.prefill_prefix_lens
        for i, L in enumerate(b.prefill_lens):
            slots.append(B.mace_kv_slot_mapping(b.prefill_block_tables[i], b.block_size, int(pfx[i]) if pfx is not None else 0, int(L)))
        for j, n in enumerate(b.decode_ctx):
            nb = -(-(int(n) + 1) // b.block_size)
            slots.append(B.mace_kv_slot_mapping(b.decode_block_tables[j][:nb], b.block_size, int(n), 1))
        self.slot_mapping_host = np.concatenate(slots).astype(np.int32) if slots else np.zeros(0, np.int32)
        self.seg_dev = up(seg)
        self.pos_dev = up(np.asarray(b.positions, dtype=np.int32))
        self.slot_dev = up(self.slot_mapping_host) if self.Ti else None
        self.bt_dev = up(np.ascontiguousarray(np.maximum(b.decode_block_tables, 0), dtype=np.int32)) if self.Td else None
        self.ctx_dev = up(np.asarray(b.decode_ctx, dtype=np.int32)) if self.Td else None
        self.head_norms = torch.zeros((self.Td, m.n_q_heads), dtype=torch.float32, device=self.dev) if self.Td else None
        pre = {}
        if pfx is not None and b.n_prefill:
            mbp = max(len(tb) for tb in b.prefill_block_tables)
            pbt = np.zeros((b.n_prefill, mbp), np.int32)
            for i, tb in enumerate(b.prefill_block_tables):
                pbt[i, :len(tb)] = tb
            pre = dict(prefill_block_tables=up(pbt), prefill_prefix_lens_host=np.asarray(pfx, np.int32),
                       prefill_prefix_lens=up(np.asarray(pfx, np.int32)), max_blocks_per_prefill=mbp)
        self.shared = getattr(b, "ft_chosen_lens", None) is not None
        if self.shared:      # one stored sequence per pair: rejected rows skip the chosen-response keys
            lo = np.asarray(b.ft_prompt_lens, dtype=np.int32)
            self.chosen_host = np.asarray(b.ft_chosen_lens, dtype=np.int32)
            self.chosen_dev = up(self.chosen_host)
            pre.update(ft_excl_lo=up(lo), ft_excl_hi=up(lo + self.chosen_host))
        self.batch = B.BatchDesc(b.n_prefill, b.n_decode, b.n_ft_seq, self.T, seg, self.seg_dev, self.pos_dev,
                                 self.slot_dev, self.bt_dev, np.asarray(b.decode_ctx, dtype=np.int32), self.ctx_dev,
                                 b.max_blocks_per_req, self.head_norms, **pre)
        self.tok_ft = up(np.asarray(b.token_ids[self.Ti:], dtype=np.int32)) if self.Tf else None
        ft_off = (seg[b.n_prefill + b.n_decode:] - self.Ti).astype(np.int32)
        self.ft_off_host = ft_off
        self.ft_off_dev = up(ft_off)
        self.prompt_host = np.asarray(b.ft_prompt_lens, dtype=np.int32)
        self.prompt_dev = up(self.prompt_host)
        self.ref_dev = up(np.asarray(wl.ref_logp, dtype=np.float32))
        self.n_pairs = b.n_ft_seq if self.shared else b.n_ft_seq // 2

        # paged cache
        cshape = (b.num_blocks, m.n_kv_heads, b.block_size, m.head_dim)
        self.cache_k = torch.zeros(cshape, dtype=self.io_dtype, device=self.dev)
        self.cache_v = torch.zeros(cshape, dtype=self.io_dtype, device=self.dev)
        self.cache = B.kv_cache_struct(self.cache_k, self.cache_v, b.num_blocks, b.block_size)
        if device_cache_seed is not None and self.Td:
            gen = torch.Generator(device=self.dev)
            gen.manual_seed(int(device_cache_seed))
            for c in (self.cache_k, self.cache_v):       # block by block to bound temporary memory
                step = max(1, (1 << 28) // (c[0].numel()))
                for b0 in range(0, c.shape[0], step):
                    c[b0:b0 + step] = torch.randn(c[b0:b0 + step].shape, generator=gen, device=self.dev, dtype=torch.float32).to(self.io_dtype)
        elif load_cache and self.Td and wl.ctx_k is not None:
            self.load_context(wl.ctx_k, wl.ctx_v)
        if load_cache and getattr(wl, "pre_k", None) is not None:
            self.load_prefix(wl.pre_k, wl.pre_v)

        # buffers
        max_ctx = int(b.decode_ctx.max()) if self.Td else 0
        self.saved = torch.empty(max(B.mace_fwd_saved_bytes(self.h, self.Tf), 256), dtype=torch.uint8, device=self.dev)
        self.ws = torch.empty(B.mace_workspace_bytes(self.h, self.T, self.Tf, self.Td, max_ctx, self.R), dtype=torch.uint8, device=self.dev)
        f32 = dict(dtype=torch.float32, device=self.dev)
        self.y = torch.empty((self.T, m.d_model), **f32)
        self.logp = torch.empty(max(2 * self.n_pairs, 1), **f32)
        self.loss_pair = torch.empty(max(self.n_pairs, 1), **f32)
        self.loss_mean = torch.empty(1, **f32)
        self.clpd = torch.empty(max(self.n_pairs, 1), **f32)
        self.win = torch.empty(max(self.n_pairs, 1), dtype=torch.int32, device=self.dev)
        self.dh = torch.empty((self.Tf, m.d_model), **f32)
        self.dE = torch.empty((m.vocab, m.d_model), **f32)
        self.dgf = torch.empty(m.d_model, **f32)
        self.dx = torch.empty((self.Tf, m.d_model), **f32)
        self.grads = {k: torch.empty(self.w[k].shape, **f32) for k in _WNAMES}
        self.g_struct = B.layer_grads_struct(self.grads)
        if self.lora is not None:
            self.lora_grads = {k: torch.empty(self.lora_dev[k].shape, **f32) for k in B._LORA_NAMES}
            self.lg_struct = B.lora_grads_struct(self.lora_grads)

    def load_context(self, ctx_k, ctx_v):
        """Place the already-cached rows of every decode request through mace_kv_cache_append."""
        b = self.wl.batch
        slots, ks, vs = [], [], []
        for j, n in enumerate(b.decode_ctx):
            n = int(n)
            if n == 0:
                continue
            nb = -(-n // b.block_size)
            slots.append(B.mace_kv_slot_mapping(b.decode_block_tables[j][:nb], b.block_size, 0, n))
            ks.append(ctx_k[j]); vs.append(ctx_v[j])
        if not slots:
            return
        sl = torch.from_numpy(np.concatenate(slots).astype(np.int32)).to(self.dev)
        k = torch.from_numpy(np.concatenate(ks).astype(np.float32)).to(self.dev).to(self.io_dtype).contiguous()
        v = torch.from_numpy(np.concatenate(vs).astype(np.float32)).to(self.dev).to(self.io_dtype).contiguous()
        B.mace_kv_cache_append(self.h, self.cache, k, v, sl, int(sl.numel()))

    def load_prefix(self, pre_k, pre_v):
        """Place the cached prefix of every prefill request through mace_kv_cache_append."""
        b = self.wl.batch
        slots, ks, vs = [], [], []
        for i, n in enumerate(b.prefill_prefix_lens):
            n = int(n)
            if n == 0:
                continue
            slots.append(B.mace_kv_slot_mapping(b.prefill_block_tables[i], b.block_size, 0, n))
            ks.append(pre_k[i]); vs.append(pre_v[i])
        if not slots:
            return
        sl = torch.from_numpy(np.concatenate(slots).astype(np.int32)).to(self.dev)
        k = torch.from_numpy(np.concatenate(ks).astype(np.float32)).to(self.dev).to(self.io_dtype).contiguous()
        v = torch.from_numpy(np.concatenate(vs).astype(np.float32)).to(self.dev).to(self.io_dtype).contiguous()
        B.mace_kv_cache_append(self.h, self.cache, k, v, sl, int(sl.numel()))

    def forward(self):
        if self.lora is not None:
            B.mace_hybrid_layer_fwd_lora(self.h, self.w_struct, self.lora, self.batch, self.cache if self.Ti else None,
                                         self.x, self.y, self.saved, self.ws)
            return
        B.mace_hybrid_layer_fwd(self.h, self.w_struct, self.batch, self.cache if self.Ti else None, self.x, self.y,
                                self.saved, self.ws)

    def dpo(self, backward: bool = True):
        y_ft = self.y[self.Ti:]
        if self.shared:
            frozen = self.lora is not None
            B.mace_dpo_logprob_loss_shared(self.h, y_ft, self.gf, self.E, self.tok_ft, self.ft_off_dev, self.ft_off_host,
                                           self.prompt_dev, self.prompt_host, self.chosen_dev, self.chosen_host, self.n_pairs,
                                           self.ref_dev, self.wl.beta, self.logp, self.loss_pair, self.loss_mean, self.clpd, self.win,
                                           self.dh if backward else None, self.dE if backward and not frozen else None,
                                           self.dgf if backward and not frozen else None, 0, self.ws)
            return
        if self.lora is not None and backward:      # frozen base model: only the row gradients are needed
            B.mace_dpo_logprob_loss(self.h, y_ft, self.gf, self.E, self.tok_ft, self.ft_off_dev, self.ft_off_host,
                                    self.prompt_dev, self.prompt_host, self.n_pairs, self.ref_dev, self.wl.beta, self.logp,
                                    self.loss_pair, self.loss_mean, self.clpd, self.win, self.dh, None, None, 0, self.ws)
            return
        B.mace_dpo_logprob_loss(self.h, y_ft, self.gf, self.E, self.tok_ft, self.ft_off_dev, self.ft_off_host,
                                self.prompt_dev, self.prompt_host, self.n_pairs, self.ref_dev, self.wl.beta, self.logp,
                                self.loss_pair, self.loss_mean, self.clpd, self.win,
                                self.dh if backward else None, self.dE if backward else None,
                                self.dgf if backward else None, 0, self.ws)

    def backward(self, dy=None):
        if self.lora is not None:
            B.mace_hybrid_layer_bwd_lora(self.h, self.w_struct, self.lora, self.batch, self.x, self.dh if dy is None else dy,
                                         self.saved, self.dx, self.lg_struct, 0, self.ws)
            return
        B.mace_hybrid_layer_bwd(self.h, self.w_struct, self.batch, self.x, self.dh if dy is None else dy, self.saved,
                                self.dx, self.g_struct, 0, self.ws)

    def step(self):
        """One pass of the whole hot path: forward of all rows, DPO head fwd+bwd, layer backward."""
        self.forward()
        if self.n_pairs:
            self.dpo(True)
            self.backward()

    def step_with_plans(self):
        """One step; returns the GEMM launch plans (binding.mace_launch_plan) of the three calls."""
        plans = {}
        self.forward()
        plans["fwd"] = B.mace_launch_plan(self.h)
        if self.n_pairs:
            self.dpo(True)
            plans["dpo"] = B.mace_launch_plan(self.h)
            self.backward()
            plans["bwd"] = B.mace_launch_plan(self.h)
        return plans

    def close(self):
        if self.h is not None:
            B.mace_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
