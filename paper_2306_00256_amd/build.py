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
SOURCES = ["api.cpp", "schedule.cpp", "chain.hip", "multi_round.hip", "mix.hip", "graph.hip", "gemv.hip", "consensus.hip", "probe.hip"]


def hipcc_path() -> str:
    for cand in (os.environ.get("HIPCC"), shutil.which("hipcc"), "/opt/rocm/bin/hipcc"):
        if cand and os.path.exists(cand):
            return cand
    raise RuntimeError("hipcc not found")


def build_library(verbose: bool = True, out: str = LIB, extra=(), jobs: int = 8) -> str:
    """Compiles every source for gfx950 (one hipcc per source, side by side) and links the shared
    library; always recompiles.  Objects go to a scratch folder next to the output and are removed."""
    import tempfile
    from concurrent.futures import ThreadPoolExecutor

    common = [
        hipcc_path(), "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
        "-x", "hip",
        # packed fp32 arithmetic stays off for all device code
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-Wall", "-Wno-unused-command-line-argument",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
        *extra,
    ]
    with tempfile.TemporaryDirectory(prefix="_build_", dir=os.path.dirname(out)) as tmp:
        objs = [os.path.join(tmp, os.path.splitext(src)[0] + ".o") for src in SOURCES]

        def compile_one(pair):
            src, obj = pair
            cmd = [*common, "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            return subprocess.run(cmd, cwd=ROOT, capture_output=True, text=True)

        with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(SOURCES)))) as pool:
            results = list(pool.map(compile_one, zip(SOURCES, objs)))
        for src, res in zip(SOURCES, results):
            noise = "is not a recognized feature for this target"     # the host pass does not know the device feature
            text = "\n".join(ln for ln in (res.stdout + res.stderr).splitlines() if noise not in ln)
            if text.strip():
                print(text, file=sys.stderr, flush=True)
            if res.returncode != 0:
                raise subprocess.CalledProcessError(res.returncode, f"hipcc -c {src}")
        link = [hipcc_path(), "--offload-arch=gfx950", "-shared", "-fPIC", *objs, "-o", out]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True, cwd=ROOT)
    return out


if __name__ == "__main__":
    build_library()
    sys.exit(0)
