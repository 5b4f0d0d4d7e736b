"""GPU parity of the adapter (LoRA) variant: forward of all rows with base + adapter, DPO head,
backward with adapter gradients only, against the oracle's adapter path - same bars as the
full-weight tests."""
import pytest

from paper_2510_03283_amd import synth
from test_gpu_parity import check_iteration, custom_workload

pytestmark = pytest.mark.gpu


def test_tiny_lora(torch_mod):
    """fp32 model: the three-pass operand path, rank below the padded width."""
    spec = synth.CONFIGS["tiny"]
    check_iteration(torch_mod, synth.make_workload("tiny"), "tiny+lora8", lora=synth.make_lora(spec, rank=8, scale=2.0))


def test_edge_lora_full_size(torch_mod):
    spec = synth.CONFIGS["edge"]
    check_iteration(torch_mod, synth.make_workload("edge"), "edge+lora16", lora=synth.make_lora(spec, rank=16, scale=2.0))


@pytest.mark.parametrize("rank,scale", [(64, 0.25), (5, 1.5)])
def test_ragged_lora(torch_mod, rank, scale):
    """Ragged batch (lengths off every tile boundary), GQA 8:2, hd 128, full and odd ranks."""
    dims = synth.ModelDims(512, 8, 2, 128, 1408, 4096, io_bf16=True)
    wl = custom_workload("ragged_lora", dims, prefill=(37, 130), decode=(5, 300), n_pairs=2, prompt=33, resp=(7, 70))
    spec = synth.ConfigSpec("ragged_lora", 77, dims, None, None, None, None, 2, 33, None, (7, 70))
    check_iteration(torch_mod, wl, f"ragged+lora{rank}", lora=synth.make_lora(spec, rank=rank, scale=scale))


def test_lora_error_paths(torch_mod):
    import torch
    from paper_2510_03283_amd import binding as B
    from paper_2510_03283_amd.harness import DeviceIteration
    spec = synth.CONFIGS["tiny"]
    wl = synth.make_workload("tiny")
    it = DeviceIteration(wl, lora=synth.make_lora(spec, rank=8))
    try:
        bad = B.lora_struct(it.lora_dev, 65, 1.0)
        with pytest.raises(B.MaceError):
            B.mace_hybrid_layer_fwd_lora(it.h, it.w_struct, bad, it.batch, it.cache, it.x, it.y, it.saved, it.ws)
        bad = B.lora_struct(it.lora_dev, 8, float("nan"))
        with pytest.raises(B.MaceError):
            B.mace_hybrid_layer_fwd_lora(it.h, it.w_struct, bad, it.batch, it.cache, it.x, it.y, it.saved, it.ws)
        torch.cuda.synchronize()
    finally:
        it.close()
