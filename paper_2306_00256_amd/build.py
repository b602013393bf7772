"""Builds libceca.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libceca.so")
SOURCES = ["api.cpp", "schedule.cpp", "chain.hip", "multi_round.hip", "mix.hip", "gemv.hip", "consensus.hip"]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose: bool = True, out: str = LIB, extra=()) -> str:
    """Compiles every source for gfx950 and links the shared library; always recompiles."""
    cmd = [
        hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
        "-x", "hip",
        # packed fp32 arithmetic stays off for all device code
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wno-unused-command-line-argument",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
        *extra,
        *[os.path.join(CSRC, s) for s in SOURCES],
        "-o", out,
    ]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, cwd=ROOT)
    return out


if __name__ == "__main__":
    build_library()
    sys.exit(0)
