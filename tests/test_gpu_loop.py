"""GPU parity of the two loop-closing entry points: next-token logits (+ greedy token) of inference
rows and the AdamW step."""
import numpy as np
import pytest

from helpers import max_abs_norm_err, run_oracle
from oracle import mace_oracle as O
from paper_2510_03283_amd import synth
from test_gpu_parity import custom_workload

pytestmark = pytest.mark.gpu


def _check_logits(torch, wl, label):
    from paper_2510_03283_amd import binding as B
    from paper_2510_03283_amd.harness import DeviceIteration
    ref = run_oracle(wl, backward=False)
    it = DeviceIteration(wl)
    try:
        it.forward()
        b = wl.batch
        rows = [int(b.seg_offsets[i + 1]) - 1 for i in range(b.n_prefill)] + list(range(it.Tp, it.Ti))   # last prefill rows, decode rows
        rows = np.array(rows, np.int32)
        n, V = len(rows), wl.dims.vocab
        logits = torch.empty((n, V), dtype=torch.float32, device="cuda")
        nxt = torch.empty(n, dtype=torch.int32, device="cuda")
        B.mace_next_token_logits(it.h, it.y, torch.from_numpy(rows).cuda(), n, it.gf, it.E, logits, nxt, it.ws)
        torch.cuda.synchronize()
        want, want_tok = O.next_token_logits(wl.dims, wl.weights, ref["y"][rows])
        got = logits.cpu().numpy()
        e = max_abs_norm_err(got, want)
        print(f"[{label}] next-token logits of {n} rows: {e:.2e}", flush=True)
        assert e <= 1e-2
        tok = nxt.cpu().numpy()
        # the decision itself is taken on the fp32 logits the library produced: exact, lowest index on ties
        assert np.array_equal(tok, np.argmax(got, axis=1))
        # and it is the oracle's token wherever the oracle's two best logits are further apart than the tolerance
        srt = np.sort(want, axis=1)
        clear = (srt[:, -1] - srt[:, -2]) > 2e-2 * np.abs(want).max()
        assert clear.any() and np.array_equal(tok[clear], want_tok[clear])
        # rows 0..n-1 without an index list
        B.mace_next_token_logits(it.h, it.y, None, 3, it.gf, it.E, logits, None, it.ws)
        torch.cuda.synchronize()
        w3, _ = O.next_token_logits(wl.dims, wl.weights, ref["y"][:3])
        assert max_abs_norm_err(logits.cpu().numpy()[:3], w3) <= 1e-2
    finally:
        it.close()


def test_next_token_logits_tiny(torch_mod):
    _check_logits(torch_mod, synth.make_workload("tiny"), "tiny")


def test_next_token_logits_bf16(torch_mod):
    dims = synth.ModelDims(512, 8, 2, 64, 1408, 8192, io_bf16=True)
    wl = custom_workload("logits", dims, prefill=(37, 130, 1), decode=(5, 300, 0, 77, 129), n_pairs=0, prompt=3, resp=(2, 9))
    _check_logits(torch_mod, wl, "bf16")


@pytest.mark.parametrize("bf", [True, False])
def test_adamw_steps(torch_mod, bf):
    import torch
    from paper_2510_03283_amd import binding as B
    h = B.mace_create(256, 4, 4, 64, 704, 2048, 1e-6, 1e4, B.MACE_BF16 if bf else B.MACE_F32)
    try:
        n = 100003                                           # ragged against the block size
        p0 = 0.02 * synth.normal(7, 90, 0, n)
        if bf:
            p0 = synth.round_to_bf16(p0.astype(np.float32)).astype(np.float64)
        lr, b1, b2, eps, wd = 1e-3, 0.9, 0.95, 1e-8, 0.1
        param = torch.from_numpy(p0.astype(np.float32)).cuda().to(torch.bfloat16 if bf else torch.float32)
        master = torch.from_numpy(p0.astype(np.float32)).cuda() if bf else None
        m = torch.zeros(n, dtype=torch.float32, device="cuda"); v = torch.zeros_like(m)
        po, mo, vo = p0.copy(), np.zeros(n), np.zeros(n)
        for step in range(1, 4):
            g = (1e-3 * synth.normal(7, 91, step * n, n)).astype(np.float32)
            B.mace_adamw_step(h, param, master, torch.from_numpy(g).cuda(), m, v, lr, b1, b2, eps, wd, step)
            torch.cuda.synchronize()
            po, mo, vo = O.adamw_step(po, g.astype(np.float64), mo, vo, step, lr, b1, b2, eps, wd)
            cur = (master if bf else param).cpu().numpy().astype(np.float64)
            assert np.max(np.abs(cur - po)) <= 2e-6 * np.max(np.abs(po)) + 1e-9, step
            assert np.max(np.abs(m.cpu().numpy() - mo)) <= 1e-6 * np.max(np.abs(mo))
            assert np.max(np.abs(v.cpu().numpy() - vo)) <= 1e-6 * np.max(np.abs(vo))
            if bf:      # the stored parameter is the round-to-nearest-even bf16 of the fp32 master, bit for bit
                want = synth.bf16_bits(synth.round_to_bf16(master.cpu().numpy()))
                got = param.view(torch.int16).cpu().numpy().view(np.uint16)
                assert np.array_equal(got, want)
        with pytest.raises(B.MaceError):
            B.mace_adamw_step(h, param, master, m, m, v, lr, b1, b2, eps, wd, 0)
    finally:
        B.mace_destroy(h)
