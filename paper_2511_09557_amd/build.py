"""Build librar.so (the C-ABI library) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "librar.so")
SOURCES = ["plan.cpp", "kernels.hip", "api.hip"]


def command(out: str = LIB) -> list[str]:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    return [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
            "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
            "-fno-gpu-flush-denormals-to-zero", "-ffp-contract=off",
            "-Wall", "-Wextra", "-Wno-unused-parameter",
            "-I", INCLUDE, "-I", CSRC, "-x", "hip",
            *[os.path.join(CSRC, s) for s in SOURCES], "-o", out]


def build_library(verbose: bool = False) -> str:
    cmd = command()
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose="-v" in sys.argv))
