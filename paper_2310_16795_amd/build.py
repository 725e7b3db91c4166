"""Build the C-ABI library (host codec + HIP kernels) for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(CSRC, "libqmoe.so")
SOURCES = [os.path.join(CSRC, "qmoe_host.cpp"), os.path.join(CSRC, "qmoe_device.hip")]


def hipcc_command(out: str = LIB) -> list[str]:
    return [
        "hipcc", "-O3", "-std=c++17", "-fPIC", "-shared", "--offload-arch=gfx950",
        # packed-fp32 instruction forms are kept out of the generated code on purpose
        "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
        "-I", os.path.join(ROOT, "include"), "-I", CSRC,
        "-o", out, *SOURCES,
    ]


def build_library(verbose: bool = False) -> str:
    cmd = hipcc_command()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    return LIB


if __name__ == "__main__":
    build_library(verbose=True)
    sys.exit(0)
