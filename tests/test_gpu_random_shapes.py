"""GPU parity on a seeded sweep of small random configurations: model widths, head layouts,
feed-forward and vocabulary sizes that are multiples of 64 but not of the GEMM tile sizes, ragged
request lengths, both storage types, both preference-pair layouts.  Every case runs the whole
iteration (forward, DPO head, backward) against the oracle at the bars of test_gpu_parity."""
import numpy as np
import pytest

from paper_2510_03283_amd import synth
from test_gpu_parity import check_iteration, custom_workload

pytestmark = pytest.mark.gpu


def draw_case(seed):
    rng = np.random.default_rng(1000 + seed)
    hd = int(rng.choice([64, 128]))
    hkv = int(rng.choice([1, 2, 4]))
    grp = int(rng.choice([1, 2, 4]))
    hq = hkv * grp
    d_model = 64 * int(rng.integers(2, 9))          # 128 .. 512, independent of hq * hd
    d_ff = 64 * int(rng.integers(3, 14))
    vocab = 64 * int(rng.integers(8, 40))
    dims = synth.ModelDims(d_model, hq, hkv, hd, d_ff, vocab, io_bf16=bool(rng.integers(0, 2)))
    prefill = [int(x) for x in rng.integers(1, 300, size=int(rng.integers(0, 4)))]
    decode = [int(x) for x in rng.integers(0, 700, size=int(rng.integers(0, 5)))]
    n_pairs = int(rng.integers(1, 4))
    prompt = int(rng.integers(1, 150))
    lo = int(rng.integers(1, 60))
    resp = (lo, lo + int(rng.integers(1, 200)))
    block_size = int(rng.choice([4, 16, 32]))
    return dims, prefill, decode, n_pairs, prompt, resp, block_size


@pytest.mark.parametrize("seed", range(10))
def test_random_configuration(torch_mod, seed):
    dims, prefill, decode, n_pairs, prompt, resp, bs = draw_case(seed)
    wl = custom_workload(f"rand{seed}", dims, prefill=prefill, decode=decode, n_pairs=n_pairs, prompt=prompt, resp=resp,
                         block_size=bs, seed=500 + seed)
    label = (f"rand{seed} d{dims.d_model} Hq{dims.n_q_heads} Hkv{dims.n_kv_heads} hd{dims.head_dim} F{dims.d_ff} V{dims.vocab} "
             f"bf{dims.io_bf16} P{prefill} D{decode} pairs{n_pairs} prompt{prompt} resp{resp} bs{bs}")
    if seed % 2:
        wl = synth.to_shared_prompt(wl)
        label += " shared"
    check_iteration(torch_mod, wl, label)
