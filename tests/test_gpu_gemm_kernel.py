"""Kernel-level parity of the dense contraction (mace_gemm_bf16) against its definition in fp64:
C = A B^T (+ A_lo B^T) (+ R), and the SwiGLU form hm = silu(G) U, for the operand layouts the iteration uses.
Sizes leave partial tiles in both directions (rows 700 = 2 * 256 + 188, columns 840 = 3 * 256 + 2 * 32 + 8),
outputs and residuals sit in buffers wider and longer than the product, and everything around the product must
come back untouched.  `kernel=1` pins the 256x256 four-wave kernel, which the launcher's cost model would only
pick for much larger problems (the full-size tests reach it on sampled outputs and on widths that are
multiples of its tile); reductions of one and two k tiles run its padded loop."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu

SENT = 12288.0      # exact in bf16


@pytest.fixture(scope="module")
def handle(torch_mod):
    from paper_2510_03283_amd import binding
    h = binding.mace_create(128, 2, 2, 64, 128, 128, 1e-5, 10000.0, 1)
    yield h
    binding.mace_destroy(h)


def bf16_of(torch, a):
    return torch.from_numpy(a.astype(np.float32)).cuda().to(torch.bfloat16)


def f64(t):
    return t.float().cpu().numpy().astype(np.float64)


def operands(torch, rng, la, lb, M, N, K):
    a = bf16_of(torch, rng.uniform(-1, 1, (M, K) if la == 0 else (K, M)))
    b = bf16_of(torch, rng.uniform(-1, 1, (N, K) if lb == 0 else (K, N)))
    A = f64(a) if la == 0 else f64(a).T
    B = f64(b) if lb == 0 else f64(b).T
    return a, b, A, B


def out_buffer(torch, rows, ld, dtype):
    return torch.full((rows, ld), SENT, dtype=dtype, device="cuda")


def check_out(c, ref, M, N, tol, what):
    got = f64(c)
    scale = max(np.abs(ref).max(), 1e-30)
    err = np.abs(got[:M, :N] - ref).max() / scale
    assert err <= tol, (what, err)
    assert np.all(got[:M, N:] == SENT) and np.all(got[M:] == SENT), (what, "wrote outside the product")


@pytest.mark.parametrize("kernel", [1, 0])
@pytest.mark.parametrize("la,lb,M,N,K", [(0, 0, 700, 840, 4160), (0, 0, 700, 840, 64), (0, 0, 300, 72, 128), (0, 1, 700, 840, 4096),
                                         (1, 1, 704, 840, 4100)])
def test_product_fp32_and_bf16(torch_mod, handle, kernel, la, lb, M, N, K):
    torch = torch_mod
    from paper_2510_03283_amd import binding
    rng = np.random.default_rng(K + 7 * M + la + 2 * lb)
    a, b, A, B = operands(torch, rng, la, lb, M, N, K)
    ref = A @ B.T
    for dtype, tol in ((torch.float32, 1e-5), (torch.bfloat16, 4e-3)):
        c = out_buffer(torch, M + 5, N + 24, dtype)
        binding.mace_gemm_bf16(handle, la, lb, M, N, K, a, b, c, ldc=N + 24, kernel=kernel)
        torch.cuda.synchronize()
        check_out(c, ref, M, N, tol, f"{la}{lb} {M}x{N}x{K} {dtype} kernel {kernel}")


@pytest.mark.parametrize("kernel", [1, 0])
@pytest.mark.parametrize("resid", ["f32", "bf16"])
def test_two_pass_with_residual(torch_mod, handle, kernel, resid):
    torch = torch_mod
    from paper_2510_03283_amd import binding
    M, N, K = 700, 840, 4096
    rng = np.random.default_rng(31 + (resid == "bf16"))
    a, b, A, B = operands(torch, rng, 0, 0, M, N, K)
    a_lo = bf16_of(torch, rng.uniform(-1, 1, (M, K)) / 256)
    ldr = N + 40
    r = torch.from_numpy(rng.uniform(-30, 30, (M + 3, ldr)).astype(np.float32)).cuda()
    if resid == "bf16":
        r = r.to(torch.bfloat16)
    ref = (A + f64(a_lo)) @ B.T + f64(r)[:M, :N]
    c = out_buffer(torch, M + 5, N + 24, torch.float32)
    binding.mace_gemm_bf16(handle, 0, 0, M, N, K, a, b, c, a_lo=a_lo, resid=r, ldc=N + 24, ldr=ldr, kernel=kernel)
    torch.cuda.synchronize()
    check_out(c, ref, M, N, 1e-5, f"two-pass + {resid} residual, kernel {kernel}")


@pytest.mark.parametrize("kernel", [1, 0])
@pytest.mark.parametrize("keep", [False, True])
def test_swiglu_form(torch_mod, handle, kernel, keep):
    """hm = silu(G) U with G = A Wg^T, U = A Wu^T; keep: the second bf16 term of hm and G | U are written too
    (what the fine-tune rows save for the backward pass)."""
    torch = torch_mod
    from paper_2510_03283_amd import binding
    M, F, K = 700, 840, 4096
    rng = np.random.default_rng(97 + keep)
    a = bf16_of(torch, rng.uniform(-1, 1, (M, K)))
    wg = bf16_of(torch, rng.uniform(-1, 1, (F, K)) / 16)
    wu = bf16_of(torch, rng.uniform(-1, 1, (F, K)) / 16)
    G, U = f64(a) @ f64(wg).T, f64(a) @ f64(wu).T
    ref = G / (1.0 + np.exp(-G)) * U
    hm = out_buffer(torch, M + 5, F, torch.bfloat16)
    lo = out_buffer(torch, M + 5, F, torch.bfloat16) if keep else None
    gu = out_buffer(torch, M + 5, 2 * F, torch.bfloat16) if keep else None
    binding.mace_gemm_bf16(handle, 0, 0, M, F, K, a, wg, hm, b_up=wu, c_lo=lo, c_gu=gu, ldc=F, swiglu=True, kernel=kernel)
    torch.cuda.synchronize()
    check_out(hm, ref, M, F, 4e-3, f"hm, kernel {kernel}")
    if keep:
        two = f64(hm) + f64(lo)
        assert np.all(f64(lo)[M:] == SENT)
        assert np.abs(two[:M] - ref).max() / np.abs(ref).max() <= 5e-5, "hm in two terms"
        check_out(gu, np.concatenate([G, U], axis=1), M, 2 * F, 4e-3, f"G | U, kernel {kernel}")


def test_swiglu_backward_form(torch_mod, handle):
    """dG | dU from dHm = dY Wd and the forward's G | U, formed in the epilogue of the product (four-wave kernel, NN form)."""
    torch = torch_mod
    from paper_2510_03283_amd import binding
    M, F, K = 700, 840, 4096
    rng = np.random.default_rng(211)
    dy = bf16_of(torch, rng.uniform(-1, 1, (M, K)))
    wd = bf16_of(torch, rng.uniform(-1, 1, (K, F)) / 16)          # [K, N]: the n-contiguous operand of the NN form
    gu = bf16_of(torch, rng.uniform(-4, 4, (M + 5, 2 * F)))
    dhm = f64(dy) @ f64(wd)
    G, U = f64(gu)[:M, :F], f64(gu)[:M, F:]
    s = 1.0 / (1.0 + np.exp(-G))
    ref = np.concatenate([dhm * U * s * (1.0 + G * (1.0 - s)), dhm * G * s], axis=1)
    dgu = out_buffer(torch, M + 5, 2 * F, torch.bfloat16)
    binding.mace_gemm_bf16(handle, 0, 1, M, F, K, dy, wd, dgu, c_gu=gu, ldc=2 * F, swiglu=2, kernel=1)
    torch.cuda.synchronize()
    check_out(dgu, ref, M, 2 * F, 4e-3, "dG | dU")
    with pytest.raises(binding.MaceError):      # only the four-wave kernel has this form
        binding.mace_gemm_bf16(handle, 0, 1, M, F, K, dy, wd, dgu, c_gu=gu, ldc=2 * F, swiglu=2, kernel=0)


@pytest.mark.parametrize("rotate", [True, False])
def test_rotary_form(torch_mod, handle, rotate):
    """The QKV product with the rotary embedding and the two-term split in its epilogue: heads of 128 columns, column
    i < 64 of a head paired with column i + 64, angles from a per-row table; 2.5 heads wide tiles and 700 rows leave
    partial tiles in both directions."""
    torch = torch_mod
    from paper_2510_03283_amd import binding
    M, N, K = 700, 640, 4096
    rng = np.random.default_rng(401 + rotate)
    a, b, A, B = operands(torch, rng, 0, 0, M, N, K)
    ang = rng.uniform(-3.0, 3.0, (M + 5, 64))
    cs = torch.from_numpy(np.stack([np.cos(ang), np.sin(ang)], axis=-1).astype(np.float32)).cuda().contiguous()
    P = (A @ B.T).reshape(M, N // 128, 2, 64)
    if rotate:
        c64, s64 = f64(cs)[:M, None, :, 0], f64(cs)[:M, None, :, 1]
        ref = np.stack([P[:, :, 0] * c64 - P[:, :, 1] * s64, P[:, :, 1] * c64 + P[:, :, 0] * s64], axis=2).reshape(M, N)
    else:
        ref = P.reshape(M, N)
    hi = out_buffer(torch, M + 5, N, torch.bfloat16)
    lo = out_buffer(torch, M + 5, N, torch.bfloat16)
    binding.mace_gemm_bf16(handle, 0, 0, M, N, K, a, b, hi, c_lo=lo, ldc=N, kernel=1, rope_cs=cs, rope_rotate=rotate)
    torch.cuda.synchronize()
    check_out(hi, ref, M, N, 4e-3, f"first term, rotate {rotate}")
    assert np.all(f64(lo)[M:] == SENT)
    two = f64(hi)[:M] + f64(lo)[:M]
    assert np.abs(two - ref).max() / np.abs(ref).max() <= 5e-5, "two terms"


@pytest.mark.parametrize("seed", range(16))
def test_random_shapes_on_the_four_wave_kernel(torch_mod, handle, seed):
    """Seeded sweep of small ragged problems pinned to the four-wave kernel: one to 600 rows, 2 to 700 columns (not
    multiples of the 32-wide accumulator blocks), one to twelve k tiles, the three layouts, both output types, either
    residual type, padded leading dimensions."""
    torch = torch_mod
    from paper_2510_03283_amd import binding
    rng = np.random.default_rng(7000 + seed)
    la, lb = [(0, 0), (0, 1), (1, 1)][int(rng.integers(0, 3))]
    M = int(rng.integers(1, 76)) * 8 if la == 1 else int(rng.integers(1, 601))
    N = int(rng.integers(1, 88)) * 8 if lb == 1 else 2 * int(rng.integers(1, 351))
    K = 64 * int(rng.integers(1, 13))
    a, b, A, B = operands(torch, rng, la, lb, M, N, K)
    ref = A @ B.T
    bf16_out = bool(rng.integers(0, 2))
    ldc = N + 2 * int(rng.integers(0, 9))
    r = None
    if not bf16_out and rng.integers(0, 2):
        r = torch.from_numpy(rng.uniform(-20, 20, (M + 2, ldc + 6)).astype(np.float32)).cuda()
        if rng.integers(0, 2):
            r = r.to(torch.bfloat16)
        ref = ref + f64(r)[:M, :N]
    c = out_buffer(torch, M + 3, ldc, torch.bfloat16 if bf16_out else torch.float32)
    binding.mace_gemm_bf16(handle, la, lb, M, N, K, a, b, c, resid=r, ldc=ldc, ldr=None if r is None else ldc + 6, kernel=1)
    torch.cuda.synchronize()
    check_out(c, ref, M, N, 4e-3 if bf16_out else 1e-5, f"seed {seed}: layouts {la}{lb}, {M}x{N}x{K}, bf16 out {bf16_out}, residual {None if r is None else r.dtype}")


def test_rejects_what_the_four_wave_kernel_cannot_do(torch_mod, handle):
    torch = torch_mod
    from paper_2510_03283_amd import binding
    a = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    b = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    c = torch.zeros((64, 66), dtype=torch.bfloat16, device="cuda")
    r = torch.zeros((64, 66), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.MaceError):      # bf16 output with a residual is not a form of that kernel
        binding.mace_gemm_bf16(handle, 0, 0, 64, 64, 64, a, b, c, resid=r, ldc=66, kernel=1)
    binding.mace_gemm_bf16(handle, 0, 0, 64, 64, 64, a, b, c, resid=r, ldc=66, kernel=0)
    torch.cuda.synchronize()
