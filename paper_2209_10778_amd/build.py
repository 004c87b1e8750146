"""Compiles libnfad.so (gfx950) in-tree with hipcc.  Run: python -m paper_2209_10778_amd.build"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRCS = [os.path.join(HERE, "csrc", f) for f in ("nfad_kernels.hip", "nfad_chain.hip")]
LIB = os.path.join(HERE, "libnfad.so")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-shared",
    # packed fp32 VALU forms are kept off on the test machines
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fno-gpu-rdc", "-Wall", "-Wno-unused-function",
]


def build(extra_flags=(), out=LIB, verbose=True) -> str:
    cmd = [HIPCC, *FLAGS, *extra_flags, "-o", out, *SRCS]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    build(sys.argv[1:])
