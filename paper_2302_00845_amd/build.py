"""Builds the HIP libraries of this package in-tree with hipcc for gfx950.

    python -m paper_2302_00845_amd.build

The shared objects are written next to the sources' package directory so that
they travel with the tree; nothing is cached elsewhere.
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libcdgrab.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 VALU forms are kept out of the generated code
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build_library(verbose: bool = True) -> str:
    src = os.path.join(CSRC, "cdgrab.hip")
    cmd = [HIPCC, *HIP_FLAGS, "-o", LIB, src]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
