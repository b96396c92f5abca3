"""Build the gfx950 shared library (libserq.so) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libserq.so")
SOURCES = ["api.hip", "quantize_act.hip", "pack.hip", "skinny.hip", "gemm_mfma.hip", "gemm_mx.hip", "skinny_mx.hip", "mx.hip", "peaks.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # kernels that take their first arguments one by one get them preloaded into SGPRs by the
    # dispatcher instead of fetching them with a scalar load (0.25 us on a 6 us decode launch)
    "-mllvm", "-amdgpu-kernarg-preload-count=12",
    "-Wno-unused-command-line-argument", "-Wno-inline-asm",
]


def build_library(verbose: bool = True, extra=()) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, *extra, "-o", LIB] + [os.path.join(CSRC, s) for s in SOURCES]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build_library(extra=sys.argv[1:])
