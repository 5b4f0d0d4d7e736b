"""GPU parity on a grouped-query layer with 128-wide heads that is large enough for the 256x256 tile: the
fine-tune rows' rotary embedding and operand split then run in the epilogue of the QKV product and the
SwiGLU backward in the epilogue of dHm = dY Wd (four-wave GEMM kernel), with column segments of three
different widths (Q: 8 heads, K and V: 2 heads each).  The launch plan is asked to confirm that these forms
ran; the whole iteration is compared element by element with the oracle at the bars of test_gpu_parity.  (The
7B-class tests reach the same code with multi-head attention and on sampled outputs.)"""
import pytest

from paper_2510_03283_amd import synth
from test_gpu_parity import check_iteration, custom_workload

pytestmark = pytest.mark.gpu


def test_gqa_layer_on_the_four_wave_forms(torch_mod):
    from paper_2510_03283_amd.harness import DeviceIteration
    dims = synth.ModelDims(1024, 8, 2, 128, 2048, 2048, io_bf16=True)
    wl = custom_workload("gqa_w4", dims, prefill=[100], decode=[40, 7], n_pairs=8, prompt=512, resp=(400, 512), block_size=16, seed=909)
    it = DeviceIteration(wl)
    try:
        plans = it.step_with_plans()
        torch_mod.cuda.synchronize()
        names_fwd = [r["name"] for r in plans["fwd"]]
        names_bwd = [r["name"] for r in plans["bwd"]]
        assert "qkv gemm + rope" in names_fwd, names_fwd
        assert "dhm gemm + swiglu bwd" in names_bwd, names_bwd
    finally:
        it.close()
    check_iteration(torch_mod, wl, "gqa d1024 Hq8 Hkv2 hd128 F2048 V2048")
