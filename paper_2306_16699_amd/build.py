"""Builds librinr.so (hipcc, gfx950) in-tree.  `python -m paper_2306_16699_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
SO = os.path.join(HERE, "librinr.so")

HIP_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-fno-gpu-rdc",
             "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
             "-Wall", "-Wno-unused-command-line-argument"]


def build(verbose: bool = False, extra=()) -> str:
    srcs = [os.path.join(CSRC, n) for n in ("rinr_api.hip", "rinr_pack.cpp", "rinr_bounds.cpp", "rinr_fit.hip", "rinr_encode.cpp")]
    cmd = ["hipcc", *HIP_FLAGS, *extra, "-o", SO, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return SO


if __name__ == "__main__":
    build(verbose=True, extra=sys.argv[1:])
