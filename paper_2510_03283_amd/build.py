"""Build the HIP library in-tree: one object per csrc/*.hip (gfx950), linked into libmace_hip.so.

Usage: python -m paper_2510_03283_amd.build
"""
from __future__ import annotations

import concurrent.futures
import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
BUILD_DIR = os.path.join(PKG_DIR, "_build")
LIB_PATH = os.path.join(PKG_DIR, "libmace_hip.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-Wall", "-Wno-unused-function",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def sources():
    return sorted(f for f in os.listdir(CSRC) if f.endswith(".hip"))


# Sources whose generated code is checked after compilation: {source: checker script in csrc/}.  The
# four-wave GEMM counts its own memory waits, so its build verifies that the compiler kept every register
# with a load in flight untouched (hipcc -save-temps leaves the gfx950 assembly beside the object).
ASM_CHECKS = {"gemm.hip": "check_w4_asm.py"}


def _compile(src: str) -> str:
    obj = os.path.join(BUILD_DIR, src[:-4] + ".o")
    cmd = [HIPCC, *FLAGS, "-c", os.path.join(CSRC, src), "-o", obj]
    if src in ASM_CHECKS:
        cmd.insert(1, "-save-temps=obj")
    r = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError(f"hipcc failed on {src}:\n{err}")
    if err.strip():
        sys.stderr.write(err + "\n")
    if src in ASM_CHECKS:
        asm = os.path.join(BUILD_DIR, src[:-4] + "-hip-amdgcn-amd-amdhsa-gfx950.s")
        c = subprocess.run([sys.executable, os.path.join(CSRC, ASM_CHECKS[src]), asm], capture_output=True, text=True)
        if c.returncode != 0:
            raise RuntimeError(f"generated-code check failed for {src}:\n{c.stdout}{c.stderr}")
    return obj


def build_library(jobs: int = 8) -> str:
    """Compile every source (always, even if a library exists) and link the shared library."""
    os.makedirs(BUILD_DIR, exist_ok=True)
    with concurrent.futures.ThreadPoolExecutor(max_workers=min(jobs, 16)) as ex:
        objs = list(ex.map(_compile, sources()))
    cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", LIB_PATH,
           "-Wl,--version-script=" + os.path.join(CSRC, "exports.map")]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("link failed:\n" + r.stderr)
    return LIB_PATH


if __name__ == "__main__":
    print(build_library())
