"""Build the gfx950 shared library (libserq.so) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys
import tempfile
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libserq.so")
SOURCES = ["api.hip", "quantize_act.hip", "pack.hip", "skinny.hip", "gemm_mfma.hip", "gemm_mx.hip", "skinny_mx.hip",
           "mx.hip", "peaks.hip", "noalloc.hip", "grouped.hip", "fp6.hip"]
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # kernels that take their first arguments one by one get them preloaded into SGPRs by the
    # dispatcher instead of fetching them with a scalar load (0.25 us on a 6 us decode launch)
    "-mllvm", "-amdgpu-kernarg-preload-count=12",
    "-Wno-unused-command-line-argument", "-Wno-inline-asm",
]


def build_library(verbose: bool = True, extra=(), jobs: int = 8) -> str:
    """Compile every source to an object file (in parallel) and link them into libserq.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    sources = list(SOURCES)
    with tempfile.TemporaryDirectory(prefix="serq_build_") as tmp:
        def compile_one(src: str) -> str:
            obj = os.path.join(tmp, src + ".o")
            cmd = [hipcc, *FLAGS, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
            if verbose:
                print(" ".join(cmd), flush=True)
            subprocess.run(cmd, check=True, stdout=subprocess.DEVNULL if not verbose else None,
                           stderr=subprocess.PIPE if not verbose else None)
            return obj

        with ThreadPoolExecutor(max_workers=max(1, min(jobs, len(sources)))) as pool:
            objs = list(pool.map(compile_one, sources))
        link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
        if verbose:
            print(" ".join(link), flush=True)
        subprocess.run(link, check=True)
    return LIB


if __name__ == "__main__":
    build_library(extra=sys.argv[1:])
