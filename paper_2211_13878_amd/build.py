"""Compile the HIP library for gfx950 (cross-compiles without a GPU).

    python -m paper_2211_13878_amd.build
"""
from __future__ import annotations

import os
import shutil
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


def check_isa_text(text: str) -> int:
    """Verify what the hand-issued scalar loads assume about the compiler's output
    (see isa_check.py); returns the number of such loads checked, raises on a violation."""
    from .isa_check import count_requests, scalar_prefetch_violations
    bad = scalar_prefetch_violations(text)
    if bad:
        lines = "\n".join(f"  {f}: load at line {a}, line {b}: {t}" for f, a, b, t in bad[:8])
        raise RuntimeError(f"{len(bad)} uses of scalar registers with a load still in flight; this build "
                           f"must not run on a GPU:\n{lines}")
    n = count_requests(text)
    if n == 0:
        raise RuntimeError("no s_load_dwordx16 found in the device code: the check is not looking at the sweep kernel")
    return n


def check_isa(extra_flags=()) -> int:
    """The same check on a fresh device-only compile (no library is produced)."""
    return check_isa_text(device_isa(extra_flags))


def compiler_id() -> str:
    """First lines of `hipcc --version`: the check's verdict holds for this compiler build only."""
    out = subprocess.check_output([HIPCC, "--version"], text=True).split("\n")
    return " | ".join(ln.strip() for ln in out[:2])


def build_library(extra_flags=(), out: str = LIB) -> str:
    """Always compiles.  The device assembly that goes INTO the library (the compiler's own
    intermediate file, kept with --save-temps) is checked before the library is put in place,
    so a library that exists at `out` has passed; it carries a stamp that says so, which the
    binding asks for when it loads it.  A violation leaves `out` untouched and raises."""
    import glob
    import hashlib
    import tempfile
    with open(SRC, "rb") as fh:
        digest = hashlib.sha256(fh.read() + " ".join([*FLAGS, *extra_flags]).encode()).hexdigest()[:16]
    stamp = f"isa-checked src+flags {digest}; {compiler_id()}"
    with tempfile.TemporaryDirectory() as d:
        tmp = os.path.join(d, "libgalvdp.so")
        cmd = [HIPCC, *FLAGS, *extra_flags, "--save-temps", f'-DGALV_DP_BUILD_STAMP="{stamp}"', "-o", tmp, SRC]
        subprocess.check_call(cmd, cwd=d)
        asm = glob.glob(os.path.join(d, "*gfx950*.s"))
        if len(asm) != 1:
            raise RuntimeError(f"expected one gfx950 assembly file among the compiler's temporaries, found {asm}")
        with open(asm[0]) as fh:
            n = check_isa_text(fh.read())
        staged = out + f".tmp{os.getpid()}"
        shutil.copyfile(tmp, staged)
        os.chmod(staged, 0o755)
    os.replace(staged, out)
    return out


if __name__ == "__main__":
    print(build_library(sys.argv[1:]))
