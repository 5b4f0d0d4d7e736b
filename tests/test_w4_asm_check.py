"""The build step that checks the generated code of the four-wave GEMM (csrc/check_w4_asm.py), on synthetic
assembly: the kernel counts its own memory waits, so the checker has to notice a register that is used while
its load is still in flight, a scratch access inside the loop and a load issued behind the loop."""
import importlib.util
import os

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2510_03283_amd", "csrc")


def _checker():
    spec = importlib.util.spec_from_file_location("check_w4_asm", os.path.join(CSRC, "check_w4_asm.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def _kernel(loop_extra="", first_wait="s_waitcnt vmcnt(1)", tail_extra=""):
    """A miniature of the kernel's shape: two loads in flight per register set, five barriers, a drain."""
    return f"""
\tbuffer_load_dwordx4 v[0:3], v20, s[0:3], s8 offen
\tbuffer_load_dwordx4 v[4:7], v20, s[0:3], s9 offen
\ts_waitcnt vmcnt(1)
\tds_write_b128 v21, v[0:3]
\tbuffer_load_dwordx4 v[0:3], v20, s[0:3], s8 offen
\ts_barrier
.LBB0_1:
\t{first_wait}
\tds_write_b128 v21, v[4:7]
\tbuffer_load_dwordx4 v[4:7], v20, s[0:3], s9 offen
\tv_mfma_f32_32x32x16_bf16 a[0:15], v[8:11], v[12:15], a[0:15]
{loop_extra}
\ts_barrier
\ts_waitcnt vmcnt(1)
\tds_write_b128 v21, v[0:3]
\tbuffer_load_dwordx4 v[0:3], v20, s[0:3], s8 offen
\ts_barrier
\ts_cbranch_scc1 .LBB0_1
\ts_waitcnt vmcnt(0)
\ts_branch .LBB0_1
.LBB0_2:
\tds_write_b128 v21, v[4:7]
\ts_barrier
\tv_mov_b32_e32 v0, v30
{tail_extra}
\ts_barrier
\tglobal_store_dword v[40:41], v0, off
\ts_endpgm
""".split("\n")


def test_clean_kernel_passes():
    ok, msg = _checker().check("k", _kernel())
    assert ok, msg


def test_register_used_before_its_load_is_waited_for():
    ok, msg = _checker().check("k", _kernel(first_wait="s_waitcnt vmcnt(2)"))
    assert not ok and "ds_write_b128 v21, v[4:7]" in msg


def test_compiler_copy_of_a_register_in_flight():
    ok, msg = _checker().check("k", _kernel(loop_extra="\tv_mov_b32_e32 v31, v5"))
    assert not ok and "v_mov_b32_e32 v31, v5" in msg


def test_scratch_access_inside_the_loop():
    ok, msg = _checker().check("k", _kernel(loop_extra="\tscratch_store_dword off, v30, off"))
    assert not ok and "scratch_store_dword" in msg


def test_load_behind_the_loop():
    ok, msg = _checker().check("k", _kernel(tail_extra="\tbuffer_load_dwordx4 v[4:7], v20, s[0:3], s9 offen"))
    assert not ok and "loads issued behind the loop" in msg


def test_generated_code_of_the_built_library_passes():
    asm = os.path.join(ROOT, "paper_2510_03283_amd", "_build", "gemm-hip-amdgcn-amd-amdhsa-gfx950.s")
    if not os.path.exists(asm):
        pytest.skip("library not built in this tree")
    assert _checker().main(asm) == 0
