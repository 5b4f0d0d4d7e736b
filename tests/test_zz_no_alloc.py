"""mace_next_token_logits_static (the entry point for callers that cannot allocate: its scratch is a
buffer built into the library) against mace_next_token_logits, through the C ABI: bit-identical
logits and tokens on two calls in a row, the second with a smaller input, plus the size limits."""
import numpy as np
import pytest

from paper_2510_03283_amd import synth

pytestmark = pytest.mark.gpu


def _hidden(torch, rows, d, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    return torch.randn((rows, d), generator=g, device="cuda", dtype=torch.float32)


def test_static_scratch_entry_point_matches_workspace_entry_point(torch_mod):
    torch = torch_mod
    from paper_2510_03283_amd import binding as B
    d, V = 2048, 32000
    h = B.mace_create(d, 32, 8, 64, 5632, V, 1e-6, 1e4, B.MACE_BF16)
    try:
        spec = synth.CONFIGS["edge"]
        E = torch.from_numpy(synth.round_to_bf16(0.02 * synth.normal(spec.seed, synth.STREAMS["E"], 0, V * d).reshape(V, d).astype(np.float32))).cuda().to(torch.bfloat16)
        gf = torch.from_numpy(synth.round_to_bf16((1.0 + 0.02 * synth.normal(spec.seed, synth.STREAMS["gf"], 0, d)).astype(np.float32))).cuda().to(torch.bfloat16)
        y = _hidden(torch, 700, d, 3)
        ws = torch.empty(B.mace_workspace_bytes(h, 700, 0, 0, 0, 0), dtype=torch.uint8, device="cuda")
        # two calls in a row on the shared buffer: 300 gathered rows, then 37 rows taken in order (the buffer
        # still holds the first call's rows beyond the 37)
        for n, with_idx in ((300, True), (37, False)):
            idx = torch.from_numpy(np.random.default_rng(n).permutation(700)[:n].astype(np.int32)).cuda() if with_idx else None
            want_l = torch.empty((n, V), dtype=torch.float32, device="cuda")
            want_t = torch.empty(n, dtype=torch.int32, device="cuda")
            got_l = torch.full((n, V), float("nan"), dtype=torch.float32, device="cuda")
            got_t = torch.full((n,), -7, dtype=torch.int32, device="cuda")
            B.mace_next_token_logits(h, y, idx, n, gf, E, want_l, want_t, ws)
            B.mace_next_token_logits_static(h, y, idx, n, gf, E, got_l, got_t)
            torch.cuda.synchronize()
            assert torch.isfinite(want_l).all()
            assert torch.equal(got_l, want_l), n            # same kernels, same launch shapes: the same bits
            assert torch.equal(got_t, want_t), n
        # limits: 4 MiB of scratch = 1024 rows of d_model 2048
        big_y = _hidden(torch, 1025, d, 4)
        out = torch.empty((1025, V), dtype=torch.float32, device="cuda")
        B.mace_next_token_logits_static(h, big_y, None, 1024, gf, E, out[:1024], None)
        torch.cuda.synchronize()
        with pytest.raises(B.MaceError, match="scratch"):
            B.mace_next_token_logits_static(h, big_y, None, 1025, gf, E, out, None)
    finally:
        B.mace_destroy(h)
    h32 = B.mace_create(256, 4, 4, 64, 704, 2048, 1e-6, 1e4, B.MACE_F32)
    try:
        with pytest.raises(B.MaceError, match="bf16"):
            B.mace_next_token_logits_static(h32, torch.zeros((2, 256), device="cuda"), None, 2, torch.ones(256, device="cuda"),
                                            torch.zeros((2048, 256), device="cuda"), torch.empty((2, 2048), device="cuda"), None)
    finally:
        B.mace_destroy(h32)
