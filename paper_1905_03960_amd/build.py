"""Build libp3.so (HIP, gfx950 only) in-tree with hipcc.

    python -m paper_1905_03960_amd.build

Flags that matter for results: -ffp-contract=off (one rounding per operation,
so the GPU reproduces the CPU checker bit for bit) and packed-fp32 instruction
selection switched off.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libp3.so")
SOURCES = ["p3_runtime.hip", "p3_drain.hip", "p3_drain_lean.hip"]
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # every atomic here is issued by one chosen lane; the wave-aggregation pass would add a
    # broadcast (and a wait for the result) right behind each of them
    "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
    "-Wall", "-Wextra", "-Wno-unused-parameter",
]


def hipcc():
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def build_library(verbose=False, extra=()):
    cmd = [hipcc(), *HIPCC_FLAGS, *extra, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           "-o", LIB, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    r = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 target feature: harmless
    err = "\n".join(l for l in r.stderr.splitlines() if "packed-fp32-ops" not in l)
    if r.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + r.stdout + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
