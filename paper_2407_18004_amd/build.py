"""Builds the gfx950 shared library in-tree with hipcc.

    python -m paper_2407_18004_amd.build

The result, libbcast_mi355x.so next to this file, is what the binding loads.
"""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "bcast_kernels.hip")
LIB = os.path.join(HERE, "libbcast_mi355x.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
    # scalar float code must not be fused into packed FP32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-command-line-argument",
]


def hipcc_path() -> str:
    found = shutil.which("hipcc")
    if found:
        return found
    cand = "/opt/rocm/bin/hipcc"
    if os.path.exists(cand):
        return cand
    raise RuntimeError("hipcc not found: the library can only be built with ROCm installed")


def build(verbose: bool = False) -> str:
    cmd = [hipcc_path(), *HIPCC_FLAGS, "-o", LIB, SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, cwd=HERE, capture_output=True, text=True)
    noise = "packed-fp32-ops"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed ({res.returncode}):\n{err}")
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
