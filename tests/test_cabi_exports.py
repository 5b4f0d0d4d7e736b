"""CPU-side checks of the boundary: the shared library loads, exports every symbol that
include/mace.h declares, and its host-only entry point (slot mapping) is integer-exact."""
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mace.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mace_[a-z_0-9]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    from paper_2510_03283_amd import binding, build
    if not os.path.exists(binding.lib_path()):
        build.build_library()
    return binding.load()


def test_every_declared_symbol_is_exported(lib):
    from paper_2510_03283_amd import binding
    syms = declared_symbols()
    assert len(syms) >= 11
    for s in syms:
        assert hasattr(lib, s), f"{s} declared in mace.h but not exported"
    assert sorted(binding.EXPORTS) == syms


def test_nothing_but_the_declared_entry_points_is_exported(lib):
    """The dynamic symbol table of the library holds the mace_* functions of the header and no internal
    launcher, hook or global."""
    import subprocess
    from paper_2510_03283_amd import binding
    out = subprocess.run(["nm", "-D", "--defined-only", binding.lib_path()], capture_output=True, text=True, check=True).stdout
    funcs = sorted(l.split()[-1] for l in out.splitlines() if l.split()[1] in "TtWw")
    assert funcs == declared_symbols(), set(funcs) ^ set(declared_symbols())


def test_slot_mapping_matches_oracle_bit_exactly(lib):
    from oracle import mace_oracle as O
    from paper_2510_03283_amd import binding as B
    rng = np.random.default_rng(0)
    for Bsz in (1, 2, 16, 64):
        for _ in range(5):
            nb = int(rng.integers(1, 40))
            bt = rng.permutation(1000)[:nb].astype(np.int32)
            start = int(rng.integers(0, nb * Bsz))
            n = int(rng.integers(0, nb * Bsz - start + 1))
            got = B.mace_kv_slot_mapping(bt, Bsz, start, n)
            assert got.dtype == np.int32
            assert np.array_equal(got.astype(np.int64), O.slot_mapping(bt, Bsz, start, n))
    # block-boundary context: the new token of a request with 32 cached tokens opens block 2
    assert list(B.mace_kv_slot_mapping(np.array([7, 3, 9], np.int32), 16, 32, 1)) == [9 * 16]


def test_slot_mapping_error_paths(lib):
    from paper_2510_03283_amd import binding as B
    with pytest.raises(B.MaceError):
        B.mace_kv_slot_mapping(np.array([1, 2], np.int32), 16, 30, 5)     # runs past the table
    with pytest.raises(B.MaceError):
        B.mace_kv_slot_mapping(np.array([1, -1], np.int32), 16, 16, 1)    # negative block id
    with pytest.raises(B.MaceError):
        B.mace_kv_slot_mapping(np.array([1, 2], np.int32), 12, 0, 1)      # block size not a power of two


def test_kv_head_budget_matches_oracle_bit_for_bit():
    """Host-side integer work: capacity split of Section 4.3, same double-precision decisions."""
    import numpy as np
    from oracle import mace_oracle as O
    from paper_2510_03283_amd import binding as B
    rng = np.random.default_rng(12)
    cases = [([1.0, 1.0, 2.0], 10), ([1.0, 1.0, 1.0], 10), ([3.0, 1.0], 8), ([5.0], 17), ([0.5, 0.25, 0.25], 1), ([2.0, 2.0], 0)]
    for _ in range(300):
        H = int(rng.integers(1, 65))
        cases.append((rng.uniform(1e-3, 9.0, H).astype(np.float32).astype(np.float64), int(rng.integers(0, 1 << 20))))
    for abar, C in cases:
        got = B.mace_kv_head_budget(abar, C)
        assert np.array_equal(got, O.head_budget(abar, C)), (abar, C)
        assert got.sum() == C
    import pytest
    with pytest.raises(B.MaceError):
        B.mace_kv_head_budget([1.0, 0.0], 5)
    with pytest.raises(B.MaceError):
        B.mace_kv_head_budget([1.0, float("nan")], 5)
