#!/usr/bin/env python3
"""Benchmark of one hybrid iteration (all hot-path steps) of the edge-small configuration on one MI355X.

A step = forward of all rows (prefill + decode + fine-tune), DPO head forward and backward, and
the layer backward of the fine-tune rows, over one synthetic mixed batch that is resident in HBM.
Prints ONE JSON line: value = rows of the batch per second over the timed steps; roofline = the
kernel class with the largest summed time among those that run alone, timed with HIP events that
the library records on the launch stream (achieved = algorithmic flops or bytes / time, against the
MI355X peak); kernel_* = per-class figures of an untimed pass in which every launch is bracketed;
cpu_baseline = the fp64 oracle timed once on the same workload on the host cores."""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "mixed-batch tokens/s per layer (prefill+decode+DPO) & % of MFMA/HBM roofline"
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0

# rocprofv3 --pmc FETCH_SIZE + WRITE_SIZE, scaled by a plain copy, bytes per launch averaged over one step's
# launches of the class: (workload, kernel class) -> bytes, from the two committed counter summaries
# (edge GEMM NT class, decode-heavy attention).  Not measured -> null.
TRAFFIC_BYTES_PER_LAUNCH = {("edge", "gemm_nt"): 5.735e8, ("7b_decode", "attn_decode"): 2.2027e10}


def cpu_baseline(wl, lora=None):
    """The oracle as it stands, timed once on the whole workload on the host cores."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import run_oracle
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    t0 = time.time()
    run_oracle(wl, backward=True, lora=lora)
    dt = time.time() - t0
    return {"value": wl.batch.n_tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"whole workload, 1 pass ({wl.batch.n_tokens} rows, {dt:.1f} s)"}


def time_extras(it, wl, torch, B, reps=10):
    """Next-token logits (last row of every prefill request + every decode row) and one AdamW step over
    the seven weight matrices of the layer, each timed with events on the stream they run on."""
    import numpy as np
    b, m = wl.batch, wl.dims
    rows = np.array([int(b.seg_offsets[i + 1]) - 1 for i in range(b.n_prefill)] + list(range(it.Tp, it.Ti)), np.int32)
    res = {}
    ev = lambda: torch.cuda.Event(enable_timing=True)
    if len(rows):
        ridx = torch.from_numpy(rows).cuda()
        logits = torch.empty((len(rows), m.vocab), dtype=torch.float32, device="cuda")
        nxt = torch.empty(len(rows), dtype=torch.int32, device="cuda")
        for _ in range(2):
            B.mace_next_token_logits(it.h, it.y, ridx, len(rows), it.gf, it.E, logits, nxt, it.ws)
        e0, e1 = ev(), ev()
        e0.record()
        for _ in range(reps):
            B.mace_next_token_logits(it.h, it.y, ridx, len(rows), it.gf, it.E, logits, nxt, it.ws)
        e1.record(); torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / reps
        # HBM-bound at this row count: E [V, d] bf16 read once + fp32 logits written once
        by = m.vocab * m.d_model * 2 + len(rows) * m.vocab * 4
        res["next_token_logits"] = {"rows": int(len(rows)), "ms": ms, "GB/s": by / ms / 1e6,
                                    "TFLOP/s": 2.0 * len(rows) * m.vocab * m.d_model / ms / 1e9}
    names = [k for k in ("wq", "wk", "wv", "wo", "wg", "wu", "wd")]
    n_el = sum(it.w[k].numel() for k in names)
    st = {k: (it.w[k].float().clone(), torch.zeros_like(it.grads[k]), torch.zeros_like(it.grads[k])) for k in names}
    def step(t):
        for k in names:
            master, mm, vv = st[k]
            B.mace_adamw_step(it.h, it.w[k], master if it.w[k].dtype != torch.float32 else None, it.grads[k], mm, vv,
                              1e-5, 0.9, 0.95, 1e-8, 0.0, t)
    step(1)
    e0, e1 = ev(), ev()
    e0.record()
    for r in range(reps):
        step(2 + r)
    e1.record(); torch.cuda.synchronize()
    ms = e0.elapsed_time(e1) / reps
    bpe = 4 * 3 + 4 * 2 + (4 + 4 + 2 + 2 if it.w["wq"].dtype != torch.float32 else 4 + 4) - (2 if it.w["wq"].dtype != torch.float32 else 0)
    # per element: read g, m, v (12 B), write m, v (8 B); bf16 model: read master 4, write master 4 + param 2; fp32 model: read 4, write 4
    res["adamw"] = {"elements": int(n_el), "ms": ms, "GB/s": n_el * bpe / ms / 1e6, "frac_of_8TB/s": n_el * bpe / ms / 1e6 / 8000.0}
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="edge", help="synthetic configuration (default: the one the metric is quoted on)")
    ap.add_argument("--variant", default="full", choices=["full", "lora"],
                    help="full: all seven weight gradients (the headline metric); lora: frozen base model, rank-16 "
                         "adapters on the attention projections, adapter gradients only")
    ap.add_argument("--prefix", type=int, default=0,
                    help="give every prefill request a cached prefix of this many tokens (multiple of the block size; "
                         "groups of four requests share the blocks of one prefix node): prefix-shared prefill")
    ap.add_argument("--shared-prompt", action="store_true",
                    help="store every preference pair once as prompt | chosen | rejected (both responses attend to one "
                         "copy of the prompt): same losses and gradients from fewer rows; `value` counts the stored rows, "
                         "`config.equivalent_tokens_per_s` the rows of the two-sequence layout the step replaces")
    ap.add_argument("--extras", action="store_true",
                    help="also time the loop-closing entry points (next-token logits of the inference rows' last tokens, "
                         "AdamW over the layer's weights) and add them to the line as `extras`")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-profile", action="store_true", help="do not bracket launches with events")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (reference dispatches for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_03283_amd import binding as B
    from paper_2510_03283_amd import synth
    from paper_2510_03283_amd.harness import DeviceIteration

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.load()   # fails loudly when the HIP library is not built
    big_cache = args.workload in ("7b", "7b_decode", "7b_ft")     # cached contexts drawn on the GPU
    if args.prefix:
        import dataclasses
        base = synth.CONFIGS[args.workload]
        if args.prefix % base.block_size or big_cache:
            print("bench.py: --prefix needs a multiple of the block size and a host-generated cache (workload edge)", file=sys.stderr)
            sys.exit(2)
        n_pre = len(base.prefill_lens) if base.prefill_lens is not None else base.prefill_draw[0]
        synth.CONFIGS[args.workload] = dataclasses.replace(base, prefill_prefix=[args.prefix] * n_pre)
    wl = synth.make_workload(args.workload, with_cache=not big_cache)
    if args.prefix:
        nb = args.prefix // wl.batch.block_size
        for i in range(wl.batch.n_prefill):          # requests 4k .. 4k+3 hang below one prefix node
            a = i - i % 4
            wl.batch.prefill_block_tables[i][:nb] = wl.batch.prefill_block_tables[a][:nb]
            wl.pre_k[i], wl.pre_v[i] = wl.pre_k[a], wl.pre_v[a]
    rows_two_seq = wl.batch.n_tokens
    if args.shared_prompt:
        wl = synth.to_shared_prompt(wl)
    lora = synth.make_lora(wl.spec, rank=16, scale=2.0) if args.variant == "lora" else None
    it = DeviceIteration(wl, device_cache_seed=wl.spec.seed if big_cache else None, lora=lora)
    if args.calib_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        it.step()
    torch.cuda.synchronize()
    # Pass 1 (untimed): every launch bracketed by events -> per-class table and the dominant class.
    # Pass 2 (the timed region): only the dominant class is bracketed, so `value` carries the cost of
    # a handful of event records per step instead of one per launch.
    prof_all, dom = {}, None
    if not args.no_profile:
        B.mace_profile_enable(it.h, True)
        for _ in range(args.steps):
            it.step()
        torch.cuda.synchronize()
        prof_all = B.mace_profile_collect(it.h)
        # classes the library runs on its side stream overlap the main chain: their event times are not
        # the kernel's own speed, so the roofline class is the largest one that runs alone
        dom = max((k for k in prof_all if prof_all[k]["launches"] and not prof_all[k]["side_launches"] and k != "misc"),
                  key=lambda k: prof_all[k]["ms"])
        B.mace_profile_enable(it.h, [dom])
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        it.step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    prof = B.mace_profile_collect(it.h) if not args.no_profile else {}
    if not args.no_profile:
        B.mace_profile_enable(it.h, False)

    ms = dt / args.steps * 1e3
    T = it.T
    out = {
        "metric": METRIC, "value": T * args.steps / dt, "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{args.workload} (BASELINE.json configs[{synth.CONFIG_ORDER.index(args.workload)}])",
                   "rows": T, "prefill_rows": it.Tp, "decode_rows": it.Td, "ft_rows": it.Tf, "loss_rows": it.R,
                   "decode_context_tokens": int(wl.batch.decode_ctx.sum()), "n_pairs": it.n_pairs,
                   "prefill_prefix_tokens": args.prefix,
                   "variant": "full fine-tune (7 weight gradients + head)" if lora is None else "LoRA rank 16 on q,k,v,o (adapter gradients only)"},
    }
    if args.shared_prompt:
        out["config"]["ft_layout"] = "shared prompt (one stored sequence per pair)"
        out["config"]["rows_two_sequence_layout"] = rows_two_seq
        out["config"]["equivalent_tokens_per_s"] = rows_two_seq * args.steps / dt
    if prof:
        e = prof[dom]
        avg_ms = e["ms"] / e["launches"]
        hbm_classes = ("attn_decode", "logsoftmax", "dlogits")      # streamed once from HBM; the rest are contractions
        if dom not in hbm_classes and e["flops"] > 0:
            ach = e["flops"] / e["launches"] / (avg_ms * 1e-3) / 1e12
            roof = {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / PEAK_BF16_TFLOPS, "traffic": TRAFFIC_BYTES_PER_LAUNCH.get((args.workload, dom)),
                    "avg_launch_ms": avg_ms, "launches_per_step": e["launches"] / args.steps}
        else:
            ach = e["bytes"] / e["launches"] / (avg_ms * 1e-3) / 1e9
            roof = {"bound": "hbm", "kernel": dom, "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": ach / PEAK_HBM_GBS, "traffic": TRAFFIC_BYTES_PER_LAUNCH.get((args.workload, dom)),
                    "avg_launch_ms": avg_ms, "launches_per_step": e["launches"] / args.steps}
        out["roofline"] = roof
        # per-class figures of the untimed all-classes pass (side-stream classes overlap the main chain)
        out["kernel_ms_per_step"] = {k: round(v["ms"] / args.steps, 4) for k, v in prof_all.items() if v["launches"]}
        out["kernel_tflops"] = {k: round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 1) for k, v in prof_all.items() if v["launches"] and v["flops"] > 0}
        out["kernel_gbps"] = {k: round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) for k, v in prof_all.items() if v["launches"] and v["bytes"] > 0}
        out["overlapped_classes"] = [k for k, v in prof_all.items() if v["side_launches"]]
    if args.extras:
        out["extras"] = time_extras(it, wl, torch, B)
    if not args.no_cpu_baseline and not big_cache:
        out["cpu_baseline"] = cpu_baseline(wl, lora)
    it.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
