"""Builds libmxq.so (hand-written HIP kernels for gfx950 + the C ABI) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

_HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(_HERE, "csrc")
LIB = os.path.join(_HERE, "libmxq.so")
SOURCES = ["mxq_api.hip", "stream_kernels.hip", "brute_kernels.hip", "aux_kernels.hip", "diag_kernels.hip"]

# No fast-math and no FMA contraction: every rounding in the kernels is written out.
# Packed-fp32 instructions are switched off for the device compiler.
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-fvisibility=hidden",
         "-ffp-contract=off", "-fno-fast-math",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def _run(cmd, verbose):
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed: " + " ".join(cmd))


def build_library(verbose: bool = False, jobs: int = 4) -> str:
    """Compiles every translation unit (in parallel) and links libmxq.so next to this file."""
    with tempfile.TemporaryDirectory(prefix="mxq_build_") as tmp:
        objs = [os.path.join(tmp, s.replace(".hip", ".o")) for s in SOURCES]
        cmds = [["hipcc", *FLAGS, "-c", os.path.join(CSRC, s), "-o", o] for s, o in zip(SOURCES, objs)]
        with ThreadPoolExecutor(max_workers=max(1, jobs)) as pool:
            list(pool.map(lambda c: _run(c, verbose), cmds))
        _run(["hipcc", "--offload-arch=gfx950", "-shared", "-fPIC", "-fvisibility=hidden", *objs, "-o", LIB],
             verbose)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
