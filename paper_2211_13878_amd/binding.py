"""Thin ctypes binding over libgalvdp.so (the C ABI declared in include/galv_dp.h).

Argument marshalling only: every step of the search runs in the library's HIP
kernels.  PyTorch is used for device memory (tensors own every buffer) and for
the current stream.  There is no CPU fallback: a missing library raises.

The module-level functions carry the C names and take device tensors; `Solver`
bundles a handle with the workspace tensor it lives in.
"""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# GALV_DP_LIB lets a developer point at another build of the same library.
LIB_PATH = os.environ.get("GALV_DP_LIB") or os.path.join(_HERE, "libgalvdp.so")

GALV_INF = 1 << 62
GALV_OK = 0
GALV_ERR_INVALID_ARG, GALV_ERR_WORKSPACE, GALV_ERR_RANGE, GALV_ERR_HIP, GALV_ERR_STATE = 1, 2, 3, 4, 5
GALV_DP_FORCE_INT64 = 1
GALV_DP_BP_U8 = 2
GALV_DP_NO_U32 = 4
GALV_DP_NO_PEEK = 8
GALV_DP_FORCE_PEEK = 16
GALV_DP_NO_PACK = 32
GALV_DP_FORCE_PACK = 64
GALV_DP_FORCE_WIDE_TILES = 128
GALV_DP_NO_WIDE_TILES = 0x2000


def GALV_DP_STREAMS(n: int) -> int:
    """Flag bits asking for n internal streams (1 = none; 0 = automatic: each solve then takes as
    many as suit the budgets that the handle's previous solve met)."""
    return int(n) << 8

GALV_INSTANCE_OK_FAST, GALV_INSTANCE_OK_INT64, GALV_INSTANCE_OK_FAST_WIDE, GALV_INSTANCE_OK_FAST_U32 = 0, 1, 2, 3
GALV_INSTANCE_OK_U32_WIDE = 4
GALV_INSTANCE_BAD_VALUE = -1

EXPORTS = ("galv_dp_workspace_bytes", "galv_dp_create", "galv_dp_solve_batched",
           "galv_dp_backtrack", "galv_dp_solve_static", "galv_dp_best_per_budget", "galv_dp_backtrack_queries",
           "galv_dp_export_tables", "galv_dp_get_status", "galv_dp_get_stats", "galv_dp_get_config", "galv_alg1_reduce",
           "galv_dp_coarsen", "galv_dp_expand_plan",
           "galv_dp_destroy", "galv_dp_last_error", "galv_dp_build_stamp")


class GalvError(RuntimeError):
    def __init__(self, code: int, message: str):
        super().__init__(f"galv_dp error {code}: {message}")
        self.code = code


class Desc(ctypes.Structure):
    _fields_ = [("n_instances", ctypes.c_int32), ("n_layers", ctypes.c_int32),
                ("n_strategies", ctypes.c_int32), ("max_budget", ctypes.c_int32),
                ("n_transition", ctypes.c_int32), ("flags", ctypes.c_uint32)]


_lib = None


def load_library() -> ctypes.CDLL:
    """Load libgalvdp.so built in-tree; fail loudly when it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(
                f"{LIB_PATH} is missing: build it with `python -m paper_2211_13878_amd.build` "
                "(there is no CPU fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        # Only a library that the package's build step produced may run on a GPU: that step
        # checks the device assembly (hand-issued scalar loads, see isa_check.py) and stamps
        # the binary; a library built any other way carries no such stamp.
        stamp = getattr(lib, "galv_dp_build_stamp", None)
        if stamp is not None:
            stamp.restype = ctypes.c_char_p
        text = stamp().decode() if stamp is not None else "no stamp"
        if not text.startswith("isa-checked "):
            raise ImportError(f"{LIB_PATH} was not produced by `python -m paper_2211_13878_amd.build` "
                              f"(build stamp: {text!r}): its device code is unverified and must not run")
        vp, i32 = ctypes.c_void_p, ctypes.c_int32
        lib.galv_dp_workspace_bytes.argtypes = [ctypes.POINTER(Desc), ctypes.POINTER(ctypes.c_size_t)]
        lib.galv_dp_create.argtypes = [ctypes.POINTER(Desc), vp, ctypes.c_size_t, ctypes.POINTER(vp)]
        lib.galv_dp_solve_batched.argtypes = [vp] * 9
        lib.galv_dp_backtrack.argtypes = [vp, vp, vp]
        lib.galv_dp_solve_static.argtypes = [ctypes.POINTER(Desc)] + [vp] * 9
        lib.galv_dp_best_per_budget.argtypes = [vp, vp, vp, vp]
        lib.galv_dp_backtrack_queries.argtypes = [vp, i32, vp, vp, vp, vp, vp]
        lib.galv_dp_export_tables.argtypes = [vp, i32, vp, vp, vp]
        lib.galv_dp_get_status.argtypes = [vp, vp, vp]
        lib.galv_dp_get_stats.argtypes = [vp, vp, vp]
        lib.galv_dp_get_config.argtypes = [vp, ctypes.POINTER(i32)]
        lib.galv_alg1_reduce.argtypes = [i32, i32, ctypes.POINTER(i32), vp, vp, i32, i32, vp, vp, vp]
        lib.galv_dp_coarsen.argtypes = [i32] * 6 + [vp] * 10
        lib.galv_dp_expand_plan.argtypes = [i32, i32, i32, vp, vp, vp]
        lib.galv_dp_destroy.argtypes = [vp]
        for name in EXPORTS[:-2]:
            getattr(lib, name).restype = ctypes.c_int
        lib.galv_dp_last_error.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def galv_dp_last_error() -> str:
    return load_library().galv_dp_last_error().decode()


def galv_dp_build_stamp() -> str:
    return load_library().galv_dp_build_stamp().decode()


def _check(code: int):
    if code != GALV_OK:
        raise GalvError(code, galv_dp_last_error())


def _dev_ptr(t, dtype, shape=None, allow_none=False):
    if t is None:
        if allow_none:
            return None
        raise GalvError(GALV_ERR_INVALID_ARG, "a required tensor is None")
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous() and t.dtype == dtype):
        raise GalvError(GALV_ERR_INVALID_ARG, f"expected a contiguous device tensor of {dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise GalvError(GALV_ERR_INVALID_ARG, f"expected shape {tuple(shape)}, got {tuple(t.shape)}")
    return ctypes.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def make_desc(B, L, S, E_max, nR=1, flags=0) -> Desc:
    return Desc(B, L, S, E_max, nR, flags)


def galv_dp_workspace_bytes(desc: Desc) -> int:
    n = ctypes.c_size_t(0)
    _check(load_library().galv_dp_workspace_bytes(ctypes.byref(desc), ctypes.byref(n)))
    return n.value


def galv_dp_create(desc: Desc, workspace: torch.Tensor) -> ctypes.c_void_p:
    h = ctypes.c_void_p(None)
    ws = _dev_ptr(workspace, torch.uint8)
    _check(load_library().galv_dp_create(ctypes.byref(desc), ws, workspace.numel(), ctypes.byref(h)))
    return h


def galv_dp_solve_batched(h, c, m, R, r_idx, budget, best_cost, best_last, stream=None):
    _check(load_library().galv_dp_solve_batched(
        h, _dev_ptr(c, torch.int64), _dev_ptr(m, torch.int32), _dev_ptr(R, torch.int64),
        _dev_ptr(r_idx, torch.int32, allow_none=True), _dev_ptr(budget, torch.int32),
        _dev_ptr(best_cost, torch.int64), _dev_ptr(best_last, torch.int32), _stream_ptr(stream)))


def galv_dp_backtrack(h, plan, stream=None):
    _check(load_library().galv_dp_backtrack(h, _dev_ptr(plan, torch.int32), _stream_ptr(stream)))


GALV_DP_STATIC_BYTES = 32 << 20


def galv_dp_solve_static(desc, c, m, R, r_idx, budget, best_cost, best_last, plan, stream=None):
    """Solve + backtrack over the library's fixed workspace; allocates nothing."""
    _check(load_library().galv_dp_solve_static(
        ctypes.byref(desc), _dev_ptr(c, torch.int64), _dev_ptr(m, torch.int32), _dev_ptr(R, torch.int64),
        _dev_ptr(r_idx, torch.int32, allow_none=True), _dev_ptr(budget, torch.int32),
        _dev_ptr(best_cost, torch.int64), _dev_ptr(best_last, torch.int32), _dev_ptr(plan, torch.int32),
        _stream_ptr(stream)))


def galv_dp_best_per_budget(h, best_cost, best_last, stream=None):
    _check(load_library().galv_dp_best_per_budget(
        h, _dev_ptr(best_cost, torch.int64), _dev_ptr(best_last, torch.int32, allow_none=True),
        _stream_ptr(stream)))


def galv_dp_backtrack_queries(h, instance, budget, cost, plan, stream=None):
    n = int(instance.numel())
    _check(load_library().galv_dp_backtrack_queries(
        h, n, _dev_ptr(instance, torch.int32, (n,)), _dev_ptr(budget, torch.int32, (n,)),
        _dev_ptr(cost, torch.int64, allow_none=True), _dev_ptr(plan, torch.int32),
        _stream_ptr(stream)))


def galv_dp_export_tables(h, instance, C_last, bp, stream=None):
    _check(load_library().galv_dp_export_tables(
        h, int(instance), _dev_ptr(C_last, torch.int64),
        _dev_ptr(bp, torch.int32, allow_none=True), _stream_ptr(stream)))


def galv_dp_get_status(h, status, stream=None):
    _check(load_library().galv_dp_get_status(h, _dev_ptr(status, torch.int32), _stream_ptr(stream)))


def galv_dp_get_stats(h, stats, stream=None):
    _check(load_library().galv_dp_get_stats(h, _dev_ptr(stats, torch.int64), _stream_ptr(stream)))


def galv_dp_get_config(h):
    """(packed table, peek, internal streams the last solve used -- before any solve: what the first
    will use --, budget columns per workgroup) as the handle chose them."""
    out = (ctypes.c_int32 * 4)()
    _check(load_library().galv_dp_get_config(h, out))
    return tuple(int(x) for x in out)


# galv_alg1_state_t as six int32 words would misread the int64 fields; it is moved as raw bytes.
ALG1_STATE_BYTES = 32


def galv_alg1_reduce(pp_degree, stage_cost, batch_size, batch_index_base, first_window, c_p, state,
                     stream=None):
    n_batch, n_pp = int(batch_size.numel()), len(pp_degree)
    arr = (ctypes.c_int32 * n_pp)(*[int(p) for p in pp_degree])
    _dev_ptr(stage_cost, torch.int64, (n_batch * sum(int(p) for p in pp_degree),))
    _check(load_library().galv_alg1_reduce(
        n_batch, n_pp, arr, _dev_ptr(stage_cost, torch.int64), _dev_ptr(batch_size, torch.int64),
        int(batch_index_base), int(bool(first_window)), _dev_ptr(c_p, torch.int64, (n_batch, n_pp)),
        _dev_ptr(state, torch.uint8, (ALG1_STATE_BYTES,)), _stream_ptr(stream)))


def galv_dp_coarsen(fuse, granularity, c, m, R, r_idx, budget, stream=None):
    """Returns (c', m', r_idx', budget') device tensors of the coarse problem."""
    B, L, S = c.shape
    nR = R.shape[1]
    Lc = (L + fuse - 1) // fuse
    _dev_ptr(m, torch.int32, (B, L, S)); _dev_ptr(R, torch.int64, (B, nR, S, S)); _dev_ptr(budget, torch.int32, (B,))
    if r_idx is not None:
        _dev_ptr(r_idx, torch.int32, (B, L))
    c2 = torch.empty((B, Lc, S), dtype=torch.int64, device=c.device)
    m2 = torch.empty((B, Lc, S), dtype=torch.int32, device=c.device)
    r2 = torch.empty((B, Lc), dtype=torch.int32, device=c.device)
    e2 = torch.empty((B,), dtype=torch.int32, device=c.device)
    _check(load_library().galv_dp_coarsen(
        B, L, S, nR, int(fuse), int(granularity), _dev_ptr(c, torch.int64), _dev_ptr(m, torch.int32),
        _dev_ptr(R, torch.int64), _dev_ptr(r_idx, torch.int32, allow_none=True), _dev_ptr(budget, torch.int32),
        _dev_ptr(c2, torch.int64), _dev_ptr(m2, torch.int32), _dev_ptr(r2, torch.int32),
        _dev_ptr(e2, torch.int32), _stream_ptr(stream)))
    return c2, m2, r2, e2


def galv_dp_expand_plan(coarse_plan, n_layers, fuse, stream=None):
    B, Lc = coarse_plan.shape
    if Lc != (n_layers + fuse - 1) // fuse:
        raise GalvError(GALV_ERR_INVALID_ARG, "coarse plan length does not match n_layers and fuse")
    plan = torch.empty((B, n_layers), dtype=torch.int32, device=coarse_plan.device)
    _check(load_library().galv_dp_expand_plan(B, int(n_layers), int(fuse), _dev_ptr(coarse_plan, torch.int32),
                                              _dev_ptr(plan, torch.int32), _stream_ptr(stream)))
    return plan


def galv_dp_destroy(h):
    _check(load_library().galv_dp_destroy(h))


class Solver:
    """A handle plus the device workspace it was created over."""

    def __init__(self, B, L, S, E_max, nR=1, flags=0, device="cuda:0"):
        self.device = torch.device(device)
        self.B, self.L, self.S, self.E_max, self.nR = B, L, S, E_max, nR
        self.desc = make_desc(B, L, S, E_max, nR, flags)
        self.workspace_bytes = galv_dp_workspace_bytes(self.desc)
        with torch.cuda.device(self.device):
            self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=self.device)
            self.handle = galv_dp_create(self.desc, self.workspace)
        self.best_cost = torch.empty(B, dtype=torch.int64, device=self.device)
        self.best_last = torch.empty(B, dtype=torch.int32, device=self.device)
        self.plan = torch.empty((B, L), dtype=torch.int32, device=self.device)
        self._inputs = None

    def solve(self, c, m, R, r_idx, budget, stream=None):
        """Enqueue the sweep; returns (best_cost[B], best_last[B]) device tensors."""
        B, L, S, nR = self.B, self.L, self.S, self.nR
        _dev_ptr(c, torch.int64, (B, L, S)); _dev_ptr(m, torch.int32, (B, L, S))
        _dev_ptr(R, torch.int64, (B, nR, S, S)); _dev_ptr(budget, torch.int32, (B,))
        if r_idx is not None:
            _dev_ptr(r_idx, torch.int32, (B, L))
        self._inputs = (c, m, R, r_idx, budget)      # keep alive for backtrack / export
        galv_dp_solve_batched(self.handle, c, m, R, r_idx, budget, self.best_cost,
                              self.best_last, stream)
        return self.best_cost, self.best_last

    def backtrack(self, stream=None):
        galv_dp_backtrack(self.handle, self.plan, stream)
        return self.plan

    def best_per_budget(self, stream=None):
        """(best_cost[B][E_max+1], best_last[B][E_max+1]) for every budget column."""
        cost = torch.empty((self.B, self.E_max + 1), dtype=torch.int64, device=self.device)
        last = torch.empty((self.B, self.E_max + 1), dtype=torch.int32, device=self.device)
        galv_dp_best_per_budget(self.handle, cost, last, stream)
        return cost, last

    def backtrack_queries(self, instance, budget, stream=None):
        """Plans for (instance, budget) pairs given as int32 device tensors: (cost[Q], plan[Q][L])."""
        q = int(instance.numel())
        cost = torch.empty(q, dtype=torch.int64, device=self.device)
        plan = torch.empty((q, self.L), dtype=torch.int32, device=self.device)
        galv_dp_backtrack_queries(self.handle, instance, budget, cost, plan, stream)
        return cost, plan

    def export_tables(self, instance, want_bp=True, stream=None):
        C_last = torch.empty((self.E_max + 1, self.S), dtype=torch.int64, device=self.device)
        bp = (torch.empty((self.L, self.E_max + 1, self.S), dtype=torch.int32, device=self.device)
              if want_bp else None)
        galv_dp_export_tables(self.handle, instance, C_last, bp, stream)
        return C_last, bp

    def status(self, stream=None):
        st = torch.empty(self.B, dtype=torch.int32, device=self.device)
        galv_dp_get_status(self.handle, st, stream)
        return st

    def stats(self, stream=None):
        """[B][3] int64: rows reduced, rows listed, rows fetched (32-bit-key instances; see galv_dp_get_stats)."""
        st = torch.empty((self.B, 3), dtype=torch.int64, device=self.device)
        galv_dp_get_stats(self.handle, st, stream)
        return st

    def config(self):
        """dict: packed, peek, streams, tile_columns (see galv_dp_get_config)."""
        return dict(zip(("packed", "peek", "streams", "tile_columns"), galv_dp_get_config(self.handle)))

    def close(self):
        """Waits for the device (a solve in flight still uses the handle's tables, streams and
        pinned word), then frees the handle."""
        if self.handle is not None:
            if torch.cuda.is_initialized():
                torch.cuda.synchronize()
            galv_dp_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def upload(w, device="cuda:0"):
    """Copy a workloads.Workload to the device: (c, m, R, r_idx, budget) tensors."""
    to = lambda a: torch.from_numpy(a).to(device)
    return to(w.c), to(w.m), to(w.R), to(w.r_idx), to(w.budget)
