"""GPU parity of prefix-shared prefill (Section 4.3): prefill requests whose leading tokens are
already cached attend to them through their block tables.  Same bars as the other iteration tests
(the whole iteration runs: decode and fine-tune rows ride along)."""
import numpy as np
import pytest

from paper_2510_03283_amd import synth
from test_gpu_parity import check_iteration

pytestmark = pytest.mark.gpu


def prefix_workload(dims, prefill, prefix, decode, n_pairs, block_size=16, share=None, seed=91):
    spec = synth.ConfigSpec("prefix", seed, dims, list(prefill), None, list(decode), None, n_pairs, 9, None, (3, 40),
                            ref_mode="len", block_size=block_size, prefill_prefix=list(prefix))
    synth.CONFIGS["prefix"] = spec
    try:
        wl = synth.make_workload("prefix")
    finally:
        del synth.CONFIGS["prefix"]
    if share:                      # request b reuses the prefix blocks (and the prefix content) of request a
        a, b = share
        nb = prefix[a] // block_size
        assert prefix[a] == prefix[b] and prefix[a] % block_size == 0
        wl.batch.prefill_block_tables[b][:nb] = wl.batch.prefill_block_tables[a][:nb]
        wl.pre_k[b], wl.pre_v[b] = wl.pre_k[a], wl.pre_v[a]
    return wl


@pytest.mark.parametrize("hq,hkv,hd", [(8, 2, 64), (4, 4, 128)])
def test_prefix_shared_prefill(torch_mod, hq, hkv, hd):
    dims = synth.ModelDims(512, hq, hkv, hd, 1408, 4096, io_bf16=True)
    # unaligned and aligned prefixes, no prefix, prefix longer than the new part, tiles with ragged tails
    wl = prefix_workload(dims, prefill=[37, 130, 64, 5, 200], prefix=[23, 64, 0, 300, 64], decode=[5, 70], n_pairs=1, share=(1, 4))
    check_iteration(torch_mod, wl, f"prefix Hq{hq} Hkv{hkv} hd{hd}")


def test_prefix_block_size_and_long_prefix(torch_mod):
    dims = synth.ModelDims(512, 4, 1, 64, 1408, 4096, io_bf16=True)
    wl = prefix_workload(dims, prefill=[1, 129], prefix=[1000, 7], decode=[], n_pairs=0, block_size=4)
    check_iteration(torch_mod, wl, "prefix B=4")


def test_prefix_needs_bf16_cache(torch_mod):
    from paper_2510_03283_amd import binding as B
    from paper_2510_03283_amd.harness import DeviceIteration
    dims = synth.ModelDims(256, 4, 4, 64, 704, 2048, io_bf16=False)
    wl = prefix_workload(dims, prefill=[10], prefix=[16], decode=[], n_pairs=0)
    it = DeviceIteration(wl)
    try:
        with pytest.raises(B.MaceError):
            it.forward()
    finally:
        it.close()
