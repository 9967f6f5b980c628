"""Compile libovggt.so (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libovggt.so")
SOURCES = ["ovggt_api.cpp", "dap_policy.cpp", "cache_kernels.hip", "select_kernels.hip", "hybrid_kernels.hip", "attn_f32.hip", "attn_bf16.hip"]
MEASURE_LIB = os.path.join(PKG, "libovggt_measure.so")       # measurement helper, a library of its own
MEASURE_SOURCES = ["measure/mfma_loop.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                       # the score tree must not fuse mul+add
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function", "-Wno-unknown-attributes",
]


def build(verbose: bool = True, extra: list[str] | None = None) -> str:
    cmd = [HIPCC, *FLAGS, *(extra or []), "-x", "hip",
           *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    cmd = [HIPCC, *FLAGS, *(extra or []), "-x", "hip",
           *[os.path.join(CSRC, s) for s in MEASURE_SOURCES], "-o", MEASURE_LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build(extra=sys.argv[1:])
