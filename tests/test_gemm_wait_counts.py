"""Host-side check of the GEMM kernel's hand-counted LDS waits (no GPU needed).

The main loop issues its MFMA fragment reads as asm and waits for them with explicit
`s_waitcnt lgkmcnt(n)`; the compiler does not know that the registers are still in flight.  This
test compiles the kernel for gfx950, walks the instruction stream of every instantiation and
checks that no MFMA follows a fragment read without such a wait in between, and that the counts
are the number of LDS read instructions of one k step (one 16-byte read per fragment of a
k-contiguous tile, two transposing reads per fragment of a row-contiguous one)."""
import os
import re
import shutil
import subprocess

import pytest

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
CSRC = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2510_03283_amd", "csrc")


@pytest.mark.skipif(not (os.path.exists(HIPCC) or shutil.which("hipcc")), reason="hipcc not available")
def test_fragment_reads_are_waited_for(tmp_path):
    out = tmp_path / "gemm.s"
    cmd = [HIPCC, "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", CSRC, "-S", "--cuda-device-only", "-o", str(out), os.path.join(CSRC, "gemm.hip")]
    subprocess.run(cmd, check=True, capture_output=True)
    lines = out.read_text().split("\n")
    starts = [i for i, l in enumerate(lines) if re.match(r"^_Z.*gemm_bf16_dl_kernel.*:", l)]
    assert len(starts) == 9, "three tile shapes x three operand layouts"
    starts.append(len(lines))
    for k in range(len(starts) - 1):
        bm, bn, wgm, wgn, la, lb = map(int, re.search(r"ILi(\d+)ELi(\d+)ELi(\d+)ELi(\d+)ELi(\d)ELi(\d)", lines[starts[k]]).groups())
        reads_per_step = (bm // wgm // 32) * (2 if la else 1) + (bn // wgn // 32) * (2 if lb else 1)
        state, waits, n_mfma = "idle", set(), 0
        for l in lines[starts[k]:starts[k + 1]]:
            t = l.strip().split()
            if not t:
                continue
            op = t[0]
            if op.startswith("ds_read"):
                state = "reads"
            elif op == "s_waitcnt" and "lgkmcnt" in l:
                if state == "reads":
                    waits.add(int(re.search(r"lgkmcnt\((\d+)\)", l).group(1)))
                    state = "waited"
            elif op.startswith("v_mfma"):
                assert state != "reads", f"kernel {bm}x{bn} layout {la}{lb}: an MFMA follows fragment reads without a wait"
                n_mfma += 1
                state = "mfma"
            elif op.startswith("scratch_"):
                raise AssertionError(f"kernel {bm}x{bn} layout {la}{lb} uses scratch memory: {l.strip()}")
        assert n_mfma > 0
        assert waits <= {0, reads_per_step}, (bm, bn, la, lb, waits, reads_per_step)
        assert reads_per_step in waits, (bm, bn, la, lb, waits)
