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


def device_isa(extra_flags=()) -> str:
    """The gfx950 assembly hipcc produces for the kernels, with the library's own flags."""
    import tempfile
    flags = [f for f in FLAGS if f not in ("-shared", "-fPIC")]
    with tempfile.TemporaryDirectory() as d:
        asm = os.path.join(d, "galv_dp.s")
        subprocess.check_call([HIPCC, *flags, *extra_flags, "-S", "--cuda-device-only", "-o", asm, SRC])
        with open(asm) as fh:
            return fh.read()


def check_isa(extra_flags=()) -> int:
    """Verify what the hand-issued scalar loads assume about the compiler's output
    (see isa_check.py); returns the number of such loads checked, raises on a violation."""
    from .isa_check import count_requests, scalar_prefetch_violations
    text = device_isa(extra_flags)
    bad = scalar_prefetch_violations(text)
    if bad:
        lines = "\n".join(f"  {f}: load at line {a}, line {b}: {t}" for f, a, b, t in bad[:8])
        raise RuntimeError(f"{len(bad)} uses of scalar registers with a load still in flight; this build "
                           f"must not run on a GPU:\n{lines}")
    n = count_requests(text)
    if n == 0:
        raise RuntimeError("no s_load_dwordx16 found in the device code: the check is not looking at the sweep kernel")
    return n


def build_library(extra_flags=(), out: str = LIB, check: bool = True) -> str:
    """Always compiles; checks the device code; replaces the library atomically."""
    if check:
        check_isa(extra_flags)
    tmp = out + f".tmp{os.getpid()}"
    cmd = [HIPCC, *FLAGS, *extra_flags, "-o", tmp, SRC]
    subprocess.check_call(cmd)
    os.replace(tmp, out)
    return out


if __name__ == "__main__":
    print(build_library(sys.argv[1:]))
