"""Execution modes of the library that must not change results: gradient accumulation, the
single-stream option, and replay of the three calls from a captured HIP graph (fork/join of the
internal side stream included)."""
import numpy as np
import pytest

from paper_2510_03283_amd import synth
from test_gpu_parity import custom_workload

pytestmark = pytest.mark.gpu


def _workload():
    dims = synth.ModelDims(512, 8, 2, 64, 1408, 4096, io_bf16=True)
    return custom_workload("modes", dims, prefill=(37, 130), decode=(5, 300), n_pairs=2, prompt=33, resp=(7, 70))


def _outputs(it):
    t = [it.y, it.logp, it.loss_pair, it.loss_mean, it.dh, it.dE, it.dgf, it.dx] + [it.grads[k] for k in sorted(it.grads)]
    return [a.clone() for a in t]


def test_accumulate_adds_to_existing_gradients(torch_mod):
    import torch
    from paper_2510_03283_amd import binding as B
    from paper_2510_03283_amd.harness import DeviceIteration
    it = DeviceIteration(_workload())
    try:
        it.step()
        torch.cuda.synchronize()
        g1 = {k: v.clone() for k, v in it.grads.items()}
        e1, f1 = it.dE.clone(), it.dgf.clone()
        y_ft = it.y[it.Ti:]
        B.mace_dpo_logprob_loss(it.h, y_ft, it.gf, it.E, it.tok_ft, it.ft_off_dev, it.ft_off_host, it.prompt_dev, it.prompt_host,
                                it.n_pairs, it.ref_dev, it.wl.beta, it.logp, it.loss_pair, it.loss_mean, it.clpd, it.win,
                                it.dh, it.dE, it.dgf, 1, it.ws)
        B.mace_hybrid_layer_bwd(it.h, it.w_struct, it.batch, it.x, it.dh, it.saved, it.dx, it.g_struct, 1, it.ws)
        torch.cuda.synchronize()
        for k in g1:
            assert torch.allclose(it.grads[k], 2 * g1[k], rtol=1e-6, atol=1e-9), k
        assert torch.allclose(it.dE, 2 * e1, rtol=1e-6, atol=1e-9) and torch.allclose(it.dgf, 2 * f1, rtol=1e-6, atol=1e-9)
    finally:
        it.close()


def test_single_stream_switch_is_bitwise_identical(torch_mod):
    import torch
    from paper_2510_03283_amd import binding as B
    from paper_2510_03283_amd.harness import DeviceIteration
    wl = _workload()
    a = DeviceIteration(wl)
    b = DeviceIteration(wl, options={B.MACE_OPT_SINGLE_STREAM: 1})
    try:
        a.step(); b.step()
        torch.cuda.synchronize()
        assert any(r["on_side_stream"] for r in B.mace_launch_plan(a.h))          # the default does use the side stream here
        assert not any(r["on_side_stream"] for r in B.mace_launch_plan(b.h))
        for u, v in zip(_outputs(a), _outputs(b)):
            assert torch.equal(u, v)
        with pytest.raises(B.MaceError):
            B.mace_set_option(a.h, 99, 1)
        with pytest.raises(B.MaceError):
            B.mace_set_option(a.h, B.MACE_OPT_DECODE_CHUNK, 1000)
    finally:
        a.close(); b.close()


def test_graph_replay_matches_eager(torch_mod):
    """The three calls captured into one HIP graph (on a side stream of the caller, as torch does) and
    replayed: every replay must reproduce the eager results bit for bit, with eager work and
    synchronisation between the replays."""
    import torch
    from paper_2510_03283_amd.harness import DeviceIteration
    it = DeviceIteration(_workload())
    try:
        it.step()                                        # eager warm-up: launch attributes are set outside the capture
        torch.cuda.synchronize()
        want = _outputs(it)
        cache0 = (it.cache_k.clone(), it.cache_v.clone())
        g = torch.cuda.CUDAGraph()
        s = torch.cuda.Stream()
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            it.step()                                    # once more on the capture stream before capturing
            torch.cuda.synchronize()
            with torch.cuda.graph(g, stream=s):
                it.step()
        torch.cuda.synchronize()
        for rep in range(3):
            for t in [it.y, it.dh, it.dE, it.dx] + list(it.grads.values()):
                t.fill_(float("nan"))                    # eager work between replays; stale results would show
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            for u, v in zip(_outputs(it), want):
                assert torch.equal(u, v), rep
            assert torch.equal(it.cache_k, cache0[0]) and torch.equal(it.cache_v, cache0[1])
    finally:
        it.close()


def test_two_pass_head_switch(torch_mod):
    """MACE_OPT_HEAD_TWO_PASS: every logit of the DPO head is formed from two-term activations;
    same bars as the default head."""
    from paper_2510_03283_amd import binding as B
    from test_gpu_parity import check_iteration
    check_iteration(torch_mod, synth.make_workload("edge", n_prefill=1, n_decode=2), "edge ft rows, two-pass head",
                    options={B.MACE_OPT_HEAD_TWO_PASS: 1})
