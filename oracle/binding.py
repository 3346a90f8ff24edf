"""ctypes loader for the C oracle (galv_oracle.c).  Test infrastructure only."""
from __future__ import annotations

import ctypes
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "galv_oracle.c")
_LIB = os.path.join(_HERE, "libgalvoracle.so")
INF = 1 << 62
_lib = None


def build(force: bool = False) -> str:
    """Compile galv_oracle.c with gcc -O2 into a shared object beside it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-Wall", "-Wextra", "-fPIC", "-shared",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        p = ctypes.c_void_p
        lib.galv_oracle_solve.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32,
                                          p, p, p, p, ctypes.c_int32, p, p, p, p, p, p]
        lib.galv_oracle_solve.restype = ctypes.c_int
        lib.galv_oracle_inf.restype = ctypes.c_int64
        assert lib.galv_oracle_inf() == INF
        _lib = lib
    return _lib


@dataclass
class OracleResult:
    best_cost: int
    best_last: int
    plan: np.ndarray            # [L] int32
    C_last: np.ndarray | None   # [budget+1][S] int64
    bp: np.ndarray | None       # [L][budget+1][S] int32
    n_tied: int


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def solve(c, m, R, r_idx, budget, *, want_C_last=False, want_bp=False) -> OracleResult:
    """One instance.  c,m: [L][S]; R: [nR][S][S] (or [S][S]); r_idx: [L] or None."""
    lib = _load()
    c = np.ascontiguousarray(c, dtype=np.int64)
    m = np.ascontiguousarray(m, dtype=np.int32)
    R = np.ascontiguousarray(R, dtype=np.int64)
    if R.ndim == 2:
        R = R[None]
    L, S = c.shape
    nR = R.shape[0]
    assert m.shape == (L, S) and R.shape == (nR, S, S)
    if r_idx is not None:
        r_idx = np.ascontiguousarray(r_idx, dtype=np.int32)
        assert r_idx.shape == (L,)
    budget = int(budget)
    best_cost = np.zeros(1, np.int64)
    best_last = np.zeros(1, np.int32)
    n_tied = np.zeros(1, np.int64)
    plan = np.zeros(L, np.int32)
    C_last = np.empty((budget + 1, S), np.int64) if want_C_last else None
    bp = np.empty((L, budget + 1, S), np.int32) if want_bp else None
    rc = lib.galv_oracle_solve(L, S, nR, _ptr(c), _ptr(m), _ptr(R), _ptr(r_idx), budget,
                               _ptr(best_cost), _ptr(best_last), _ptr(plan), _ptr(C_last),
                               _ptr(bp), _ptr(n_tied))
    if rc != 0:
        raise RuntimeError(f"galv_oracle_solve failed with {rc}")
    return OracleResult(int(best_cost[0]), int(best_last[0]), plan, C_last, bp, int(n_tied[0]))


def solve_workload(w, instances=None, threads: int = 1, **kw) -> list[OracleResult]:
    """Solve instances of a workload one by one (optionally one per thread)."""
    ids = list(range(w.B)) if instances is None else list(instances)

    def one(b):
        c, m, R, r_idx, budget = w.instance(b)
        return solve(c, m, R, r_idx, budget, **kw)

    if threads <= 1:
        return [one(b) for b in ids]
    with ThreadPoolExecutor(max_workers=threads) as ex:
        return list(ex.map(one, ids))
