"""Algorithm 1 (paper section 3.3, "Optimization Workflow") on top of the batched solver.

The paper's loop nest is batch size -> pipeline degree P -> stage, one dynamic
program per stage.  Here a WINDOW of consecutive batch sizes is searched at
once: for each P one call of galv_dp_solve_batched solves all (batch size,
stage) instances of the window, their optima land in one device array, and
galv_alg1_reduce does the sums over stages, the minimum over P and the
throughput scan with its Out-Of-Memory stop on the device.  The host reads the
32-byte state once per window to learn whether to go on.  Batch sizes past the
stopping one are searched speculatively and ignored, so the result is that of
the sequential loop.  The solves of the different pipeline degrees are independent and run
on a stream each; every window ends with a host synchronisation, which is also what keeps
the window's device buffers alive long enough.

Host code here only marshals: it asks the cost model for tables, pads stages of
unequal length, and decodes the result.  Stage lengths differ by at most one
(layers are dealt as evenly as possible, the first L mod P stages take the extra
one); a short stage gets one trailing layer whose only usable strategy is index
0 at zero time, zero memory and zero transition cost, which leaves its optimum
unchanged.
"""
from __future__ import annotations

import struct
from dataclasses import dataclass
from fractions import Fraction

import numpy as np
import torch

from . import binding
from .strategies import group_strategies


@dataclass
class Alg1Result:
    throughput: Fraction          # batch / cost; 0 when even the first batch size does not fit
    batch: int | None
    pp: int | None
    cost: int | None
    plans: list | None            # per stage: list of strategy indices, one per layer of the stage
    n_explored: int
    stopped: bool                 # True: ended at an Out-Of-Memory batch size; False: ran out of batch sizes
    c_p: np.ndarray               # [n batch sizes searched][n degrees] time costs (GALV_INF = does not fit)


def pipeline_partition(n_layers: int, pp: int):
    q, r = divmod(n_layers, pp)
    bounds = [i * q + min(i, r) for i in range(pp + 1)]
    return list(zip(bounds[:-1], bounds[1:]))


def strategy_counts(n_devices: int, prune_dp_sdp: bool = True) -> dict:
    return {1 << k: len(group_strategies(n_devices >> k, prune_dp_sdp))
            for k in range(n_devices.bit_length())}


_streams = {}


def _stream(device, key):
    """Streams are kept for the life of the process: creating one costs far more than a small solve."""
    k = (str(device), key)
    if k not in _streams:
        _streams[k] = torch.cuda.Stream(device=device)
    return _streams[k]


class _StageBatch:
    """Solver and staging buffers for one pipeline degree and one window length."""

    def __init__(self, model, pp, window, budget, device):
        self.pp, self.window = pp, window
        self.cuts = pipeline_partition(model.n_layers, pp)
        self.Ls = max(hi - lo for lo, hi in self.cuts)
        self.S = model.n_strategies[pp]
        B = window * pp
        self.solver = binding.Solver(B, self.Ls, self.S, budget, nR=2, device=device)
        self.c = np.zeros((B, self.Ls, self.S), np.int64)
        self.m = np.zeros((B, self.Ls, self.S), np.int32)
        self.R = np.zeros((B, 2, self.S, self.S), np.int64)        # matrix 1 stays zero: padding
        self.r_idx = np.zeros((B, self.Ls), np.int32)
        self.budget = torch.full((B,), budget, dtype=torch.int32, device=device)
        unusable = np.int32(budget + 1)
        for st, (lo, hi) in enumerate(self.cuts):
            n = hi - lo
            if n < self.Ls:
                self.m[st::pp, n:, 1:] = unusable
                self.r_idx[st::pp, n:] = 1
        self.stream = _stream(device, pp)                  # the degrees' solves are independent: one stream each

    def fill(self, model, batch_sizes):
        for ib, batch in enumerate(batch_sizes):
            for st, (lo, hi) in enumerate(self.cuts):
                c, m, R = model.stage_tables(batch, self.pp, lo, hi)
                i = ib * self.pp + st
                self.c[i, :hi - lo], self.m[i, :hi - lo], self.R[i, 0] = c, m, R

    def solve_into(self, stage_cost, device):
        """Upload and solve on this degree's stream, ordered after the caller's current stream."""
        main = torch.cuda.current_stream(device)
        self.stream.wait_stream(main)
        with torch.cuda.stream(self.stream):
            to = lambda a: torch.from_numpy(a).to(device)
            self.dev = (to(self.c), to(self.m), to(self.R), to(self.r_idx), self.budget)
            s = self.solver
            s._inputs = self.dev
            binding.galv_dp_solve_batched(s.handle, *self.dev, stage_cost, s.best_last)


def optimize(model, n_devices: int, budget: int, batch_sizes, window: int = 8,
             device="cuda:0") -> Alg1Result:
    """Largest throughput B / C_opt over `batch_sizes` (ascending) until the first that fits nowhere."""
    device = torch.device(device)
    if not 0 <= budget < np.iinfo(np.int32).max:
        raise ValueError("budget must be in [0, 2^31 - 2]")
    batch_sizes = [int(b) for b in batch_sizes]
    degrees = [1 << k for k in range(n_devices.bit_length()) if (1 << k) <= model.n_layers]
    skipped = n_devices.bit_length() - len(degrees)      # degrees deeper than the layer count never fit
    stages = [_StageBatch(model, pp, window, budget, device) for pp in degrees]
    state = torch.zeros(binding.ALG1_STATE_BYTES, dtype=torch.uint8, device=device)
    c_p_rows, best_plans = [], None
    best_index, stopped, n_explored = -1, False, 0
    batch = cost = pp_index = None
    for base in range(0, len(batch_sizes), window):
        win = batch_sizes[base:base + window]
        n = len(win)
        padded = win + [win[-1]] * (window - n)           # a short last window repeats its last size
        stage_cost = torch.empty(window * sum(degrees), dtype=torch.int64, device=device)
        off = 0
        for sb in stages:
            sb.fill(model, padded)
            sb.solve_into(stage_cost[off:off + window * sb.pp], device)
            off += window * sb.pp
        for sb in stages:                                  # join: the reduction reads every degree's optima
            torch.cuda.current_stream(device).wait_stream(sb.stream)
        c_p = torch.empty((window, len(degrees)), dtype=torch.int64, device=device)
        bs = torch.tensor(padded, dtype=torch.int64, device=device)
        if n < window:                                    # scan only the real sizes of a short last window
            parts, off = [], 0
            for sb in stages:
                parts.append(stage_cost[off:off + window * sb.pp][:n * sb.pp])
                off += window * sb.pp
            stage_cost, bs, c_p = torch.cat(parts), bs[:n].clone(), c_p[:n]
        binding.galv_alg1_reduce(degrees, stage_cost, bs, base, base == 0, c_p, state)
        batch, cost, pp_index, batch_index, stop_flag, n_explored = struct.unpack(
            "<qqiiii", state.cpu().numpy().tobytes())
        c_p_rows.append(c_p.cpu().numpy())
        if batch_index >= base and batch_index != best_index:
            best_index = batch_index
            sb = stages[pp_index]
            ib = batch_index - base
            q = torch.arange(ib * sb.pp, (ib + 1) * sb.pp, dtype=torch.int32, device=device)
            _, plan = sb.solver.backtrack_queries(q, sb.budget[:sb.pp].clone())
            plan = plan.cpu().numpy()
            best_plans = [plan[st, :hi - lo].tolist() for st, (lo, hi) in enumerate(sb.cuts)]
        if stop_flag:
            stopped = True
            break
    c_p_all = np.concatenate(c_p_rows) if c_p_rows else np.zeros((0, len(degrees)), np.int64)
    if skipped:
        c_p_all = np.concatenate([c_p_all, np.full((len(c_p_all), skipped), binding.GALV_INF)], axis=1)
    c_p_all = c_p_all[:n_explored + (1 if stopped else 0)]
    for sb in stages:
        sb.solver.close()
    if best_index < 0:
        return Alg1Result(Fraction(0), None, None, None, None, n_explored, stopped, c_p_all)
    return Alg1Result(Fraction(batch, cost) if cost else Fraction(0), batch, degrees[pp_index], cost,
                      best_plans, n_explored, stopped, c_p_all)
