"""Compile the HIP sources into paper_2509_15038_amd/libcurdkv.so for gfx950.

    python -m paper_2509_15038_amd.build

hipcc cross-compiles without a GPU.  Nothing is built lazily at import time:
tests, the smoke check and the benchmark load the library this step left here.
"""

from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
LIB = os.path.join(HERE, "libcurdkv.so")
SOURCES = ["curdkv_api.hip", "scores_kernels.hip", "select_kernels.hip", "compact_kernels.hip", "fused_kernel.hip", "adaptive_kernels.hip",
           "sketch_host.cpp"]


def build(verbose: bool = True) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
           "-fno-gpu-rdc", "-Wall", "-Wno-unused-function",
           # packed fp32 VALU forms are switched off for all device code
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-I", os.path.join(ROOT, "include"), "-I", os.path.join(HERE, "csrc")]
    cmd += ["-x", "hip"] + [os.path.join(HERE, "csrc", s) for s in SOURCES]
    cmd += ["-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build()
    print("built", LIB)
    sys.exit(0)
