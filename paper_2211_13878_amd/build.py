"""Compile the HIP library for gfx950 (cross-compiles without a GPU).

    python -m paper_2211_13878_amd.build
"""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "csrc", "galv_dp.hip")
LIB = os.path.join(HERE, "libgalvdp.so")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # No NaN is ever produced (keys are non-negative integers or +inf, and +inf is
    # never subtracted), so the minimum needs no quieting of its operands.
    "-fno-honor-nans",
    "-Wall", "-Wextra", "-Wno-unused-command-line-argument",
]


def build_library(extra_flags=(), out: str = LIB) -> str:
    """Always compiles; replaces the library atomically."""
    tmp = out + f".tmp{os.getpid()}"
    cmd = [HIPCC, *FLAGS, *extra_flags, "-o", tmp, SRC]
    subprocess.check_call(cmd)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build_library(sys.argv[1:]))
