#!/usr/bin/env python3
"""Benchmark of one hybrid iteration (all hot-path steps) on one MI355X.

Headline workload: `7b_ft`, the largest single-GPU configuration (fine-tune-heavy 7B-class layer,
66,576 rows); `--workload` selects another one.  A step = forward of all rows (prefill + decode +
fine-tune), DPO head forward and backward, and the layer backward of the fine-tune rows, over one
synthetic mixed batch that is resident in HBM.  Prints ONE JSON line:

  value        rows of the batch per second over the K timed steps (one host bracket around all of
               them, synchronised on both sides); ms_per_step_median / _min / _max are per-step
               times from a pair of events around every step of the same region
  roofline     the kernel class with the largest summed time among those that run alone on the
               caller's stream, timed inside the timed region with HIP events that the library
               records on the launch stream: achieved = algorithmic flops (or bytes) / time against
               the MI355X peak; traffic is read from the tracked counter summary under profiles/
               when that summary was made from the kernel source as it is now, else null
  kernel_*     per-class figures of an untimed pass in which every launch is bracketed;
               class_frac = each class's fraction of its own roofline (MFMA or HBM peak)
  per_config   the same figures for the other bf16 configurations (shorter runs)
  cpu_baseline the fp64 oracle timed on the host cores: the whole workload where that takes seconds,
               else a request-subsampled batch (1 prefill + 1 decode + 1 pair, per-request shapes
               unchanged); rows per second is intensive, so the sub-batch figure stands for the
               workload."""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import re
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

METRIC = "mixed-batch tokens/s per layer (prefill+decode+DPO) & % of MFMA/HBM roofline"
PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA peak
PEAK_HBM_GBS = 8000.0
HEADLINE = "7b_ft"
BIG = ("7b", "7b_decode", "7b_ft")          # cached contexts drawn on the GPU; oracle timed on a sub-batch
HBM_CLASSES = ("attn_decode", "logsoftmax", "dlogits")      # streamed once from HBM; the other timed classes are contractions
# kernel class -> the source file whose hash a counter summary must carry to be quoted
GEMM_SRC = "gemm.hip+gemm_w4.h"      # several files: the hash is taken over their concatenation
CLASS_SOURCE = {"gemm_nt": GEMM_SRC, "gemm_nn": GEMM_SRC, "gemm_tn": GEMM_SRC, "attn_decode": "attn_decode.hip",
                "attn_fwd_prefill": "attn_fwd.hip", "attn_fwd_ft": "attn_fwd.hip", "attn_bwd": "attn_bwd.hip",
                "logsoftmax": "dpo_head.hip", "dlogits": "dpo_head.hip"}


def traffic_from_profiles(workload, kernel):
    """Bytes past the XCD L2s per launch of `kernel` in `workload`, from the tracked rocprofv3 counter
    summary profiles/bench_<workload>_<kernel>_hbm_traffic.md - only if the summary names the sha256 of
    the kernel source it was measured on and that source is unchanged.  Returns (bytes or None, note)."""
    path = os.path.join("profiles", f"bench_{workload}_{kernel}_hbm_traffic.md")
    full = os.path.join(ROOT, path)
    src = CLASS_SOURCE.get(kernel)
    if not os.path.exists(full) or src is None:
        return None, f"{path}: no counter summary"
    text = open(full).read()
    mt = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", text)
    mh = re.search(r"kernel_source_sha256:\s*([0-9a-f]{64})", text)
    if not mt or not mh:
        return None, f"{path}: summary carries no traffic_bytes_per_launch / kernel_source_sha256 line"
    now = hashlib.sha256(b"".join(open(os.path.join(ROOT, "paper_2510_03283_amd", "csrc", f), "rb").read() for f in src.split("+"))).hexdigest()
    if now != mh.group(1):
        return None, f"{path}: measured on another version of {src} (sha256 {mh.group(1)[:12]}.., now {now[:12]}..)"
    return float(mt.group(1)), f"{path} (csrc/{src} sha256 {now[:12]}..)"


def cpu_baseline(wl_name, wl, lora, weights):
    """The oracle as it stands, timed once on the host cores (whole workload, or a request-subsampled
    batch of the 7B-class workloads)."""
    sys.path.insert(0, os.path.join(ROOT, "tests"))
    from helpers import run_oracle
    from paper_2510_03283_amd import synth
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    if wl_name in BIG:
        b = wl.batch
        sub = synth.make_workload(wl_name, n_prefill=min(1, b.n_prefill), n_decode=min(1, b.n_decode), n_pairs=1, weights=weights)
        what = (f"request-subsampled batch of {wl_name}: {sub.batch.n_prefill} prefill + {sub.batch.n_decode} decode request(s) + 1 pair, "
                f"per-request shapes unchanged")
    else:
        sub, what = wl, "whole workload"
    t0 = time.time()
    run_oracle(sub, backward=True, lora=lora)
    dt = time.time() - t0
    return {"value": sub.batch.n_tokens / dt, "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{what}, 1 pass ({sub.batch.n_tokens} rows, {dt:.1f} s)"}


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


def class_fractions(prof):
    """Fraction of its own roofline for every timed class that has an algorithmic count."""
    out = {}
    for k, v in prof.items():
        if not v["launches"] or v["ms"] <= 0:
            continue
        if k in HBM_CLASSES and v["bytes"] > 0:
            out[k] = round(v["bytes"] / (v["ms"] * 1e-3) / 1e9 / PEAK_HBM_GBS, 4)
        elif v["flops"] > 0:
            out[k] = round(v["flops"] / (v["ms"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS, 4)
    return out


def run_workload(name, steps, warmup, args, torch, B, synth, weights=None, headline=True):
    """Build `name`, run warm-up, the all-classes pass and the timed region; returns (result dict, objects
    the caller may still need)."""
    from paper_2510_03283_amd.harness import DeviceIteration
    big_cache = name in BIG
    if args.prefix and headline:
        import dataclasses
        base = synth.CONFIGS[name]
        if args.prefix % base.block_size or big_cache:
            print("bench.py: --prefix needs a multiple of the block size and a host-generated cache (workload edge)", file=sys.stderr)
            sys.exit(2)
        n_pre = len(base.prefill_lens) if base.prefill_lens is not None else base.prefill_draw[0]
        synth.CONFIGS[name] = dataclasses.replace(base, prefill_prefix=[args.prefix] * n_pre)
    wl = synth.make_workload(name, with_cache=not big_cache, weights=weights)
    if args.prefix and headline:
        nb = args.prefix // wl.batch.block_size
        for i in range(wl.batch.n_prefill):          # requests 4k .. 4k+3 hang below one prefix node
            a = i - i % 4
            wl.batch.prefill_block_tables[i][:nb] = wl.batch.prefill_block_tables[a][:nb]
            wl.pre_k[i], wl.pre_v[i] = wl.pre_k[a], wl.pre_v[a]
    rows_two_seq = wl.batch.n_tokens
    if args.shared_prompt and headline:
        wl = synth.to_shared_prompt(wl)
    lora = synth.make_lora(wl.spec, rank=16, scale=2.0) if (args.variant == "lora" and headline) else None
    it = DeviceIteration(wl, device_cache_seed=wl.spec.seed if big_cache else None, lora=lora)
    if args.calib_copy and headline:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")      # 1 GiB read + 1 GiB written per copy
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    for _ in range(warmup):
        it.step()
    torch.cuda.synchronize()
    # Pass 1 (untimed): every launch bracketed by events -> per-class table and the dominant class.
    # Pass 2 (the timed region): only the dominant class is bracketed, so `value` carries the cost of
    # a handful of event records per step instead of one per launch.
    prof_all, dom = {}, None
    if not args.no_profile:
        B.mace_profile_enable(it.h, True)
        for _ in range(steps):
            it.step()
        torch.cuda.synchronize()
        prof_all = B.mace_profile_collect(it.h)
        # classes the library runs on its side stream overlap the main chain: their event times are not
        # the kernel's own speed, so the roofline class is the largest one that runs alone
        dom = max((k for k in prof_all if prof_all[k]["launches"] and not prof_all[k]["side_launches"] and k != "misc"),
                  key=lambda k: prof_all[k]["ms"])
        B.mace_profile_enable(it.h, [dom])
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for a, b in ev:
        a.record()
        it.step()
        b.record()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    per_step = [a.elapsed_time(b) for a, b in ev]
    prof = B.mace_profile_collect(it.h) if not args.no_profile else {}
    if not args.no_profile:
        B.mace_profile_enable(it.h, False)

    T = it.T
    res = {"ms_per_step": dt / steps * 1e3, "tokens_per_s": T * steps / dt, "steps": steps, "warmup": warmup,
           "ms_per_step_median": statistics.median(per_step), "ms_per_step_min": min(per_step), "ms_per_step_max": max(per_step),
           "config": {"workload": f"{name} (BASELINE.json configs[{synth.CONFIG_ORDER.index(name)}])",
                      "rows": T, "prefill_rows": it.Tp, "decode_rows": it.Td, "ft_rows": it.Tf, "loss_rows": it.R,
                      "decode_context_tokens": int(wl.batch.decode_ctx.sum()), "n_pairs": it.n_pairs}}
    if it.Td:
        m = wl.dims
        kv = (int(wl.batch.decode_ctx.sum()) + it.Td) * 2 * m.n_kv_heads * m.head_dim * 2
        res["config"]["decode_kv_bytes"] = kv
        # the 256 MB last-level cache can hold a small cache between steps: say so instead of quoting > HBM figures blindly
        res["config"]["decode_kv_fits_last_level_cache"] = bool(kv < 256e6)
    if headline:
        res["config"]["prefill_prefix_tokens"] = args.prefix
        res["config"]["variant"] = ("full fine-tune (7 weight gradients + head)" if lora is None
                                    else "LoRA rank 16 on q,k,v,o (adapter gradients only)")
        if args.shared_prompt:
            res["config"]["ft_layout"] = "shared prompt (one stored sequence per pair)"
            res["config"]["rows_two_sequence_layout"] = rows_two_seq
            res["config"]["equivalent_tokens_per_s"] = rows_two_seq * steps / dt
    if prof:
        e = prof[dom]
        avg_ms = e["ms"] / e["launches"]
        traffic, note = traffic_from_profiles(name, dom)
        if dom not in HBM_CLASSES and e["flops"] > 0:
            ach = e["flops"] / e["launches"] / (avg_ms * 1e-3) / 1e12
            roof = {"bound": "mfma", "kernel": dom, "achieved": ach, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                    "frac": ach / PEAK_BF16_TFLOPS}
        else:
            ach = e["bytes"] / e["launches"] / (avg_ms * 1e-3) / 1e9
            roof = {"bound": "hbm", "kernel": dom, "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                    "frac": ach / PEAK_HBM_GBS}
        roof.update({"traffic": traffic, "traffic_source": note, "avg_launch_ms": avg_ms, "launches_per_step": e["launches"] / steps})
        res["roofline"] = roof
        # per-class figures of the untimed all-classes pass (side-stream classes overlap the main chain)
        res["kernel_ms_per_step"] = {k: round(v["ms"] / steps, 4) for k, v in prof_all.items() if v["launches"]}
        res["kernel_tflops"] = {k: round(v["flops"] / (v["ms"] * 1e-3) / 1e12, 1) for k, v in prof_all.items() if v["launches"] and v["flops"] > 0}
        res["kernel_gbps"] = {k: round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) for k, v in prof_all.items() if v["launches"] and v["bytes"] > 0}
        res["class_frac"] = class_fractions(prof_all)
        res["overlapped_classes"] = [k for k, v in prof_all.items() if v["side_launches"]]
    return res, it, wl, lora


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default=HEADLINE, help="synthetic configuration (default: the largest single-GPU one)")
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
    ap.add_argument("--no-per-config", action="store_true", help="skip the short runs of the other bf16 configurations")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run three plain 1 GiB device copies (reference dispatches for scaling rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2510_03283_amd import binding as B
    from paper_2510_03283_amd import synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.load()   # fails loudly when the HIP library is not built
    if args.workload not in synth.CONFIGS:
        print(f"bench.py: unknown workload {args.workload}", file=sys.stderr)
        sys.exit(2)
    weights = synth.make_weights(synth.CONFIGS[args.workload])
    res, it, wl, lora = run_workload(args.workload, args.steps, args.warmup, args, torch, B, synth, weights=weights)
    out = {
        "metric": METRIC, "value": res["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": res["ms_per_step"], "ms_per_step_median": res["ms_per_step_median"],
        "ms_per_step_min": res["ms_per_step_min"], "ms_per_step_max": res["ms_per_step_max"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": res["config"],
    }
    for k in ("roofline", "kernel_ms_per_step", "kernel_tflops", "kernel_gbps", "class_frac", "overlapped_classes"):
        if k in res:
            out[k] = res[k]
    if args.extras:
        out["extras"] = time_extras(it, wl, torch, B)
    it.close()
    del it
    torch.cuda.empty_cache()
    plain = args.variant == "full" and not args.prefix and not args.shared_prompt
    if not args.no_per_config and not args.no_profile and plain and args.workload == HEADLINE:
        # the other bf16 configurations, shorter runs; the 7B-class ones reuse the weights drawn for the headline
        # workload (same shapes and distribution; their own seeds are what the parity tests use)
        per = {}
        for name in ("edge", "7b", "7b_decode"):
            w = weights if name in BIG else None
            r, it2, _, _ = run_workload(name, 10, 2, args, torch, B, synth, weights=w, headline=False)
            it2.close()
            del it2
            torch.cuda.empty_cache()
            rf = r["roofline"]
            per[name] = {"ms_per_step": round(r["ms_per_step"], 4), "ms_per_step_median": round(r["ms_per_step_median"], 4),
                         "tokens_per_s": round(r["tokens_per_s"], 1), "rows": r["config"]["rows"],
                         "dominant_class": rf["kernel"], "dominant_frac": round(rf["frac"], 4), "dominant_bound": rf["bound"],
                         "class_frac": r["class_frac"], "kernel_ms_per_step": r["kernel_ms_per_step"]}
            if "decode_kv_fits_last_level_cache" in r["config"]:
                per[name]["decode_kv_fits_last_level_cache"] = r["config"]["decode_kv_fits_last_level_cache"]
        out["per_config"] = per
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload, wl, lora, weights)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
