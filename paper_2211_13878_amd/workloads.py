"""Seeded synthetic inputs for the plan-search dynamic program.

This module only draws numbers.  It holds none of the method's arithmetic
(no recurrence, no min, no backtrack) so that both the CPU oracle's tests and
the HIP path can be fed the very same arrays.

An instance of the search problem (paper section 3.3, "Dynamic Programming
Search", Eq. 1) is: per-layer execution times c(l, s), per-layer memory use
O(l, s) (called m here), transformation costs R(l, s_prev, s_cur) between
neighbouring layers, and a device memory budget E.  A *workload* is a batch of
B such instances with common L (layers), S (strategies), E_max (largest
budget, in memory units) and nR (number of distinct transition matrices).

Array contract (all C-contiguous):
    c      [B][L][S]      int64   c(l, s) >= 0
    m      [B][L][S]      int32   m(l, s) >= 0 ; m > budget  => (l, s) infeasible
    R      [B][nR][S][S]  int64   R[k][s_prev][s_cur] >= 0
    r_idx  [B][L]         int32   which R matrix enters layer l (l = 0 unused)
    budget [B]            int32   0 <= budget[b] <= E_max

The five named configurations mimic the shapes of the paper's workloads
(Table 2: 32/48/128-layer models, a 24+24 encoder-decoder; section 3.2: 22
candidate strategies on 8 GPUs; Fig. 5: search time up to 96 layers) with
drawn values, since the paper's profiled costs are not published.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class Workload:
    name: str
    B: int
    L: int
    S: int
    E_max: int
    nR: int
    c: np.ndarray
    m: np.ndarray
    R: np.ndarray
    r_idx: np.ndarray
    budget: np.ndarray
    notes: dict = field(default_factory=dict)

    def instance(self, b: int):
        """Arrays of one instance: (c[L,S], m[L,S], R[nR,S,S], r_idx[L], budget)."""
        return (self.c[b], self.m[b], self.R[b], self.r_idx[b], int(self.budget[b]))

    def nominal_cell_updates(self) -> int:
        """The metric's count: sum over instances of L * E_b * S^2."""
        return int(sum(self.L * int(e) * self.S * self.S for e in self.budget))

    def exact_candidates(self) -> int:
        """Exact number of (l, e, s, s') candidates: (L-1) * (E_b+1) * S^2."""
        return int(sum((self.L - 1) * (int(e) + 1) * self.S * self.S for e in self.budget))

    def n_states(self) -> int:
        """Table cells: sum over instances of L * (E_b+1) * S."""
        return int(sum(self.L * (int(e) + 1) * self.S for e in self.budget))


def _off_diagonal(rng: np.random.Generator, S: int, hi: int) -> np.ndarray:
    """S x S matrix, i.i.d. integers in [0, hi] per ordered pair, zero diagonal."""
    R = rng.integers(0, hi + 1, size=(S, S), dtype=np.int64)
    R[np.arange(S), np.arange(S)] = 0
    return R


def _jittered(rng: np.random.Generator, base: np.ndarray, L: int, scale: np.ndarray) -> np.ndarray:
    """Per-layer copies of base[s] times scale[l] with +-5 % uniform jitter, rounded."""
    u = rng.uniform(-0.05, 0.05, size=(L, base.shape[0]))
    return np.rint(base[None, :] * scale[:, None] * (1.0 + u)).astype(np.int64)


def _stack(name, L, S, E_max, nR, per_instance, budgets, notes=None) -> Workload:
    B = len(per_instance)
    c = np.ascontiguousarray(np.stack([p[0] for p in per_instance]).astype(np.int64))
    m = np.ascontiguousarray(np.stack([p[1] for p in per_instance]).astype(np.int32))
    R = np.ascontiguousarray(np.stack([p[2] for p in per_instance]).astype(np.int64))
    r_idx = np.ascontiguousarray(np.stack([p[3] for p in per_instance]).astype(np.int32))
    budget = np.ascontiguousarray(np.asarray(budgets, dtype=np.int32))
    assert c.shape == (B, L, S) and m.shape == (B, L, S)
    assert R.shape == (B, nR, S, S) and r_idx.shape == (B, L) and budget.shape == (B,)
    return Workload(name, B, L, S, E_max, nR, c, m, R, r_idx, budget, notes or {})


def _identical_layer_instance(rng, L, S, E_max, m_lo, m_hi, c_lo, c_hi, r_hi, infeasible,
                              layer_scale):
    base_m = rng.integers(m_lo, m_hi + 1, size=S).astype(np.float64)
    base_c = rng.integers(c_lo, c_hi + 1, size=S).astype(np.float64)
    m = _jittered(rng, base_m, L, layer_scale)
    c = _jittered(rng, base_c, L, layer_scale)
    R = _off_diagonal(rng, S, r_hi)
    mask = rng.random(size=(L, S)) < infeasible
    m[mask] = E_max + 1
    return c, m, R


def config(index: int, n_instances: int | None = None) -> Workload:
    """Build named configuration `index` (0..4).

    `n_instances` truncates the batch (the first instances keep their seeds
    and their budgets) so that tests can run a prefix of a large batch.
    Seeds: numpy default_rng(1000 * index + instance); configuration 0 uses 0.
    """
    if index == 0:
        L, S, E = 4, 6, 256
        rng = np.random.default_rng(0)
        m = rng.integers(1, 32 + 1, size=(L, S))
        c = rng.integers(1000, 100000 + 1, size=(L, S))
        R = _off_diagonal(rng, S, 20000)
        inst = [(c, m, R[None], np.zeros(L, np.int32))]
        return _stack("tiny", L, S, E, 1, inst, [E])

    if index == 1:
        B, L, S, E = 8, 32, 22, 16384
        B = B if n_instances is None else min(B, n_instances)
        inst = []
        for b in range(B):
            rng = np.random.default_rng(1000 * index + b)
            c, m, R = _identical_layer_instance(rng, L, S, E, 64, 1024, 10_000, 1_000_000,
                                                50_000, 0.10, np.ones(L))
            inst.append((c, m, R[None], np.zeros(L, np.int32)))
        return _stack("bert_huge_like", L, S, E, 1, inst, [E] * B)

    if index == 2:
        B, L, S, E = 32, 48, 22, 24576
        B = B if n_instances is None else min(B, n_instances)
        scale = np.where(np.arange(L) >= 24, 1.5, 1.0)
        inst = []
        for b in range(B):
            rng = np.random.default_rng(1000 * index + b)
            c, m, R = _identical_layer_instance(rng, L, S, E, 64, 1024, 10_000, 1_000_000,
                                                50_000, 0.10, scale)
            r_idx = np.zeros(L, np.int32)
            r_idx[24] = 1
            inst.append((c, m, np.stack([R, 2 * R]), r_idx))
        return _stack("t5_like", L, S, E, 2, inst, [E] * B)

    if index == 3:
        B_full, L, S, E = 64, 96, 44, 32768
        budgets = np.rint(np.linspace(8192, 32768, B_full)).astype(np.int64)
        B = B_full if n_instances is None else min(B_full, n_instances)
        inst = []
        for b in range(B):
            rng = np.random.default_rng(1000 * index + b)
            c, m, R = _identical_layer_instance(rng, L, S, E, 32, 2048, 10_000, 1_000_000,
                                                100_000, 0.05, np.ones(L))
            inst.append((c, m, R[None], np.zeros(L, np.int32)))
        return _stack("gpt3_depth", L, S, E, 1, inst, budgets[:B])

    if index == 4:
        B, L, S, E = 16, 128, 128, 65536
        B = B if n_instances is None else min(B, n_instances)
        inst = []
        n_copied = 0
        for b in range(B):
            rng = np.random.default_rng(1000 * index + b)
            m = rng.integers(16, 4096 + 1, size=(L, S))
            c = rng.integers(1_000, 10_000_000 + 1, size=(L, S))
            R = _off_diagonal(rng, S, 1_000_000)
            # Injected ties: two strategy pairs (a, b) where b duplicates a in R
            # and, on ~64 % of the layers, in (c, m) -> about 1 % of the (l, s)
            # cells have an exact twin, so inner minima have equal candidates.
            picks = rng.choice(S, size=4, replace=False)
            for a, d in (sorted(picks[:2]), sorted(picks[2:])):
                R[d, :] = R[a, :]
                R[:, d] = R[:, a]
                R[a, d] = R[d, a] = 0
                R[a, a] = R[d, d] = 0
                rows = rng.random(size=L) < 0.64
                c[rows, d] = c[rows, a]
                m[rows, d] = m[rows, a]
                n_copied += int(rows.sum())
            inst.append((c, m, R[None], np.zeros(L, np.int32)))
        return _stack("stress", L, S, E, 1, inst, [E] * B, {"tie_cells": n_copied})

    raise ValueError(f"no configuration {index}")


N_CONFIGS = 5


def random_workload(seed: int, B: int, L: int, S: int, E_max: int, *, nR: int = 1,
                    m_range=(0, 8), c_range=(0, 9), r_range=(0, 9), infeasible: float = 0.0,
                    zero_diagonal: bool = True, budgets=None, name: str = "random") -> Workload:
    """Small i.i.d. workloads for parity and edge-case tests.

    Narrow value ranges force many equal candidates (tie-break coverage);
    m may be 0; `infeasible` marks that fraction of (l, s) with m = E_max + 1;
    budgets default to uniform draws in [0, E_max].
    """
    rng = np.random.default_rng(seed)
    inst = []
    for _ in range(B):
        m = rng.integers(m_range[0], m_range[1] + 1, size=(L, S))
        c = rng.integers(c_range[0], c_range[1] + 1, size=(L, S))
        R = rng.integers(r_range[0], r_range[1] + 1, size=(nR, S, S), dtype=np.int64)
        if zero_diagonal:
            R[:, np.arange(S), np.arange(S)] = 0
        m[rng.random(size=(L, S)) < infeasible] = E_max + 1
        r_idx = rng.integers(0, nR, size=L).astype(np.int32)
        inst.append((c, m, R, r_idx))
    if budgets is None:
        budgets = rng.integers(0, E_max + 1, size=B)
    return _stack(name, L, S, E_max, nR, inst, budgets)


class Alg1Model:
    """Seeded stand-in for the paper's cost estimator (section 3.4), as Algorithm 1 consumes it.

    For a batch size B, a pipeline degree P and a contiguous range of layers it
    returns the tables of one stage's search: c(l, s), m(l, s) and R(s', s) over
    the S_P strategies of a group of N / P devices.  Values are affine in B with
    drawn coefficients: time grows with B, so does memory (activations), faster
    strategies need more memory, a layer needs P times more memory per device on
    a group that is P times smaller, and each degree has its own speed factor.  `n_strategies` maps each P to S_P (the caller counts
    the decision trees; this class only draws numbers).
    """

    def __init__(self, seed: int, n_layers: int, n_devices: int, n_strategies: dict,
                 time_scale: int = 400, mem_fixed: int = 20, mem_per_sample: int = 4):
        self.n_layers, self.n_devices = n_layers, n_devices
        self.n_strategies = dict(n_strategies)
        rng = np.random.default_rng(seed)
        self._coef = {}
        for pp in sorted(self.n_strategies):
            S = self.n_strategies[pp]
            speed = rng.uniform(1.0, 4.0, size=(n_layers, S))
            f_pp = rng.uniform(0.7, 1.3)
            alpha = np.rint(time_scale * f_pp / speed * rng.uniform(0.9, 1.1, size=(n_layers, S)))
            beta = rng.integers(0, 5 * time_scale, size=(n_layers, S))
            mu = np.rint(mem_fixed * pp * speed)
            nu = np.rint(mem_per_sample * pp * speed)
            rho = rng.integers(0, time_scale // 2, size=(S, S))
            np.fill_diagonal(rho, 0)
            self._coef[pp] = (alpha.astype(np.int64), beta.astype(np.int64), mu.astype(np.int64),
                              nu.astype(np.int64), rho.astype(np.int64))

    def stage_tables(self, batch: int, pp: int, lo: int, hi: int):
        """(c[hi-lo][S] int64, m[hi-lo][S] int32, R[S][S] int64) of layers lo..hi-1."""
        alpha, beta, mu, nu, rho = self._coef[pp]
        c = alpha[lo:hi] * batch + beta[lo:hi]
        m = np.minimum(mu[lo:hi] + nu[lo:hi] * batch, np.iinfo(np.int32).max).astype(np.int32)
        return np.ascontiguousarray(c), np.ascontiguousarray(m), np.ascontiguousarray(rho * batch)
