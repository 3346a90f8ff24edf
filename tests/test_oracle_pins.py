"""Pins for the CPU oracle (no GPU): the serial layer recurrence is checked
against things that do not depend on it.

  * enumeration of all S^L plans (the plain definition, paper section 3.3)
    on configuration 0 and on hundreds of random tiny instances, comparing
    cost AND plan (ties: smallest plan read from the last layer);
  * textbook special cases written here with numpy: zero transition cost
    reduces to a multiple-choice knapsack, an unbinding budget reduces to a
    shortest path on the L x S trellis, both to a sum of per-layer minima;
    S = 1; L = 1; a budget below the sum of per-layer minimum memories;
  * invariants that follow from the optimal-substructure argument of the same
    section: the table is non-increasing in the budget, the returned plan
    re-evaluates to the returned cost and fits the budget, a table solved for
    budget E contains the answer for every smaller budget.
"""
import os

import numpy as np
import pytest

import oracle
from oracle.bruteforce import brute_force, brute_force_cells, plan_cost, plan_memory
from paper_2211_13878_amd import workloads

INF = oracle.INF
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _check_plan(c, m, R, r_idx, budget, res):
    """The plan re-evaluated by the plain definition equals the reported optimum."""
    if res.best_cost == INF:
        assert res.best_last == -1 and (res.plan == -1).all()
        return
    plan = [int(s) for s in res.plan]
    assert all(0 <= s < c.shape[1] for s in plan)
    assert plan[-1] == res.best_last
    assert plan_cost(c, R, r_idx, plan) == res.best_cost
    assert plan_memory(m, plan) <= budget


# ---------------------------------------------------------------- enumeration

def test_config0_matches_golden_enumeration():
    lines = [ln.split() for ln in open(os.path.join(GOLDEN, "config0_enumeration.txt"))
             if not ln.startswith("#")]
    gold = {ln[0]: [int(x) for x in ln[1:]] for ln in lines}
    w = workloads.config(0)
    res = oracle.solve(*w.instance(0))
    assert res.best_cost == gold["cost"][0]
    assert list(res.plan) == gold["plan"]
    # and the enumeration itself, re-run now
    cost, plan = brute_force(*w.instance(0))
    assert (cost, plan) == (gold["cost"][0], gold["plan"])


@pytest.mark.parametrize("seed", range(6))
def test_every_table_cell_vs_enumeration(seed):
    """The GPU parity tests compare whole tables with the oracle's, so the oracle's cells are
    pinned one by one: C[L-1][e][s] is the cheapest partial plan that ends in s within e units,
    the back-pointer of (l, e, s) the lowest former strategy that attains the cell's minimum,
    and the tie count the number of cells with several such strategies — all by enumeration of
    partial plans.  Narrow value ranges give many ties; m = 0, unusable cells, two asymmetric
    matrices with a non-zero diagonal."""
    rng = np.random.default_rng(700 + seed)
    for _ in range(6):
        L, S = int(rng.integers(1, 5)), int(rng.integers(1, 5))
        E = int(rng.integers(0, 11))
        w = workloads.random_workload(int(rng.integers(1 << 30)), 1, L, S, E, nR=2, m_range=(0, 4),
                                      c_range=(0, 3), r_range=(0, 2), infeasible=0.15,
                                      zero_diagonal=False, budgets=[E])
        c, m, R, r_idx, budget = w.instance(0)
        C, bp, n_tied = brute_force_cells(c, m, R, r_idx, budget)
        res = oracle.solve(c, m, R, r_idx, budget, want_C_last=True, want_bp=True)
        assert res.C_last.tolist() == C[L - 1]
        assert res.bp.tolist() == bp
        assert res.n_tied == n_tied


def test_tie_count_on_a_hand_made_case():
    """Two layers, three strategies, no memory pressure: cell (1, e, s) sees the candidates
    c(0, s') + R(s', s).  With c(0) = [5, 5, 7] and R = 0 except R[0][2] = 1, strategies 0
    and 1 tie between s' = 0 and 1 (both 5) while strategy 2 is won by s' = 1 alone: two tied
    cells of three per budget column."""
    c = np.array([[5, 5, 7], [1, 1, 1]], np.int64)
    m = np.zeros((2, 3), np.int32)
    R = np.array([[[0, 0, 1], [0, 0, 0], [0, 0, 0]]], np.int64)
    res = oracle.solve(c, m, R, None, 3, want_bp=True, want_C_last=True)
    assert res.n_tied == 2 * 4                       # budget columns 0..3
    assert res.bp[1].tolist() == [[0, 0, 1]] * 4 and res.C_last.tolist() == [[6, 6, 6]] * 4


@pytest.mark.parametrize("seed", range(12))
def test_random_tiny_vs_enumeration(seed):
    """25 instances per seed: narrow value ranges (many ties), m = 0 allowed,
    budget 0 allowed, infeasible cells, several asymmetric transition matrices
    with non-zero diagonal."""
    rng = np.random.default_rng(seed)
    L = int(rng.integers(1, 6))
    S = int(rng.integers(1, 5))
    E = int(rng.integers(0, 14))
    nR = int(rng.integers(1, 3))
    w = workloads.random_workload(100 + seed, 25, L, S, E, nR=nR, m_range=(0, 5),
                                  c_range=(0, 3), r_range=(0, 3),
                                  infeasible=0.1 * (seed % 3), zero_diagonal=bool(seed % 2))
    n_inf = 0
    for b in range(w.B):
        c, m, R, r_idx, budget = w.instance(b)
        res = oracle.solve(c, m, R, r_idx, budget)
        cost, plan = brute_force(c, m, R, r_idx, budget)
        assert res.best_cost == cost, (seed, b)
        assert [int(s) for s in res.plan] == plan, (seed, b)
        _check_plan(c, m, R, r_idx, budget, res)
        n_inf += cost == INF
    assert n_inf < w.B or E < 3  # not all degenerate


def test_wide_values_vs_enumeration():
    """Wider value ranges (no accidental ties), S up to 6, L up to 5."""
    for seed in range(6):
        w = workloads.random_workload(500 + seed, 4, 5, 6 - seed % 2, 40, m_range=(1, 12),
                                      c_range=(1000, 100000), r_range=(0, 20000))
        for b in range(w.B):
            inst = w.instance(b)
            res = oracle.solve(*inst)
            cost, plan = brute_force(*inst)
            assert (res.best_cost, [int(s) for s in res.plan]) == (cost, plan)


def test_transition_matrix_orientation():
    """R[former][current]: a one-directional cheap transition decides the plan."""
    c = np.zeros((2, 2), np.int64)
    m = np.zeros((2, 2), np.int32)
    R = np.array([[[5, 1], [7, 5]]], np.int64)   # only 0 -> 1 is cheap
    res = oracle.solve(c, m, R, None, 0)
    assert res.best_cost == 1 and list(res.plan) == [0, 1]
    res = oracle.solve(c, m, np.transpose(R, (0, 2, 1)).copy(), None, 0)
    assert res.best_cost == 1 and list(res.plan) == [1, 0]


def test_first_layer_pays_no_transition():
    c = np.array([[3, 4]], np.int64)
    m = np.array([[1, 1]], np.int32)
    R = np.array([[[100, 100], [100, 100]]], np.int64)
    res = oracle.solve(c, m, R, None, 1)
    assert res.best_cost == 3 and list(res.plan) == [0]
    c2 = np.array([[3, 4], [1, 1]], np.int64)
    m2 = np.array([[1, 1], [0, 0]], np.int32)
    assert oracle.solve(c2, m2, R, None, 1).best_cost == 3 + 1 + 100


def test_per_layer_transition_selector():
    c = np.zeros((3, 2), np.int64)
    m = np.zeros((3, 2), np.int32)
    R = np.array([[[9, 9], [9, 9]], [[1, 2], [3, 4]]], np.int64)
    assert oracle.solve(c, m, R, np.array([0, 0, 1], np.int32), 0).best_cost == 9 + 1
    assert oracle.solve(c, m, R, np.array([1, 1, 1], np.int32), 0).best_cost == 1 + 1
    assert oracle.solve(c, m, R, None, 0).best_cost == 18


def test_lowest_index_tie_break():
    """All plans cost the same: every index must come out 0; with the budget
    only admitting strategy 1 on the first layer, the rest stays 0."""
    L, S = 4, 3
    c = np.full((L, S), 7, np.int64)
    m = np.ones((L, S), np.int32)
    R = np.zeros((1, S, S), np.int64)
    res = oracle.solve(c, m, R, None, 10, want_bp=True)
    assert list(res.plan) == [0] * L and res.best_cost == 28 and res.n_tied > 0
    m[0] = [5, 1, 5]
    res = oracle.solve(c, m, R, None, 4)
    assert list(res.plan) == [1, 0, 0, 0]


def test_inclusive_budget_and_infinity():
    c = np.array([[1, 2], [1, 2]], np.int64)
    m = np.array([[2, 1], [2, 1]], np.int32)
    R = np.zeros((1, 2, 2), np.int64)
    assert oracle.solve(c, m, R, None, 4).best_cost == 2          # exactly fits
    assert oracle.solve(c, m, R, None, 3).best_cost == 3
    assert oracle.solve(c, m, R, None, 2).best_cost == 4
    res = oracle.solve(c, m, R, None, 1, want_C_last=True, want_bp=True)
    assert res.best_cost == INF and res.best_last == -1 and list(res.plan) == [-1, -1]
    assert (res.C_last == INF).all() and (res.bp == -1).all()


def test_huge_memory_value_is_just_infeasible():
    c = np.array([[1, 2], [1, 2]], np.int64)
    m = np.array([[2**31 - 1, 1], [2**31 - 1, 1]], np.int32)
    R = np.zeros((1, 2, 2), np.int64)
    res = oracle.solve(c, m, R, None, 5)
    assert res.best_cost == 4 and list(res.plan) == [1, 1]


# ---------------------------------------------------------- textbook reductions

def _knapsack(c, m, budget):
    """Multiple-choice knapsack, K[l][e] = min_s K[l-1][e - m(l,s)] + c(l,s)."""
    L, S = c.shape
    big = np.iinfo(np.int64).max // 4
    K = np.zeros(budget + 1, np.int64)
    for l in range(L):
        new = np.full(budget + 1, big, np.int64)
        for s in range(S):
            w = int(m[l, s])
            if w <= budget:
                new[w:] = np.minimum(new[w:], K[:budget + 1 - w] + c[l, s])
        K = np.minimum(new, big)
    return K


def _trellis_shortest_path(c, R, r_idx):
    V = c[0].astype(np.int64)
    for l in range(1, c.shape[0]):
        V = c[l] + (V[:, None] + R[r_idx[l]]).min(axis=0)
    return int(V.min())


@pytest.mark.parametrize("seed", range(5))
def test_zero_transition_is_multiple_choice_knapsack(seed):
    w = workloads.random_workload(700 + seed, 3, 9, 7, 300, m_range=(0, 60),
                                  c_range=(1, 1000), r_range=(0, 0), infeasible=0.05)
    for b in range(w.B):
        c, m, R, r_idx, _ = w.instance(b)
        res = oracle.solve(c, m, R, r_idx, w.E_max, want_C_last=True)
        K = _knapsack(c, m.astype(np.int64), w.E_max)
        got = res.C_last.min(axis=1)
        want = np.where(K >= np.iinfo(np.int64).max // 8, INF, K)
        assert (got == want).all()


@pytest.mark.parametrize("seed", range(5))
def test_unbinding_budget_is_trellis_shortest_path(seed):
    w = workloads.random_workload(800 + seed, 3, 12, 9, 12 * 20, nR=2, m_range=(0, 20),
                                  c_range=(0, 5000), r_range=(0, 3000), zero_diagonal=False,
                                  budgets=[12 * 20] * 3)
    for b in range(w.B):
        c, m, R, r_idx, budget = w.instance(b)
        res = oracle.solve(c, m, R, r_idx, budget)
        assert res.best_cost == _trellis_shortest_path(c, R, r_idx)
        _check_plan(c, m, R, r_idx, budget, res)


def test_closed_forms():
    rng = np.random.default_rng(3)
    L, S = 10, 5
    c = rng.integers(1, 100, size=(L, S)).astype(np.int64)
    m = rng.integers(1, 9, size=(L, S)).astype(np.int32)
    R0 = np.zeros((1, S, S), np.int64)
    R = rng.integers(0, 50, size=(1, S, S)).astype(np.int64)
    # no transition cost and no binding budget: sum of per-layer minima
    assert oracle.solve(c, m, R0, None, int(m.max(axis=1).sum())).best_cost == c.min(axis=1).sum()
    # budget below the sum of per-layer minimum memories: infinity; at it: finite
    low = int(m.min(axis=1).sum())
    assert oracle.solve(c, m, R, None, low - 1).best_cost == INF
    assert oracle.solve(c, m, R, None, low).best_cost < INF
    # a single strategy: the plan is forced
    c1, m1, R1 = c[:, :1].copy(), m[:, :1].copy(), np.array([[[4]]], np.int64)
    want = int(c1.sum()) + 4 * (L - 1)
    assert oracle.solve(c1, m1, R1, None, int(m1.sum())).best_cost == want
    assert oracle.solve(c1, m1, R1, None, int(m1.sum()) - 1).best_cost == INF
    # a single layer: cheapest strategy that fits
    for budget in range(0, 10):
        fits = m[0] <= budget
        want = int(c[0][fits].min()) if fits.any() else INF
        res = oracle.solve(c[:1], m[:1], R, None, budget)
        assert res.best_cost == want
        if fits.any():
            assert res.best_last == int(np.flatnonzero(fits & (c[0] == want))[0])


# ------------------------------------------------------------------ invariants

def _table_invariants(c, m, R, r_idx, budget, res):
    C, bp = res.C_last, res.bp
    L, S = c.shape
    assert (C[1:] <= C[:-1]).all()                       # non-increasing in e
    assert (bp[0] == -1).all()                           # layer 0 has no former layer
    assert (bp < S).all() and (bp >= -1).all()
    if L > 1:
        assert ((bp[L - 1] >= 0) == (C < INF)).all()     # reachable <=> has a pointer
    assert res.best_cost == C[budget].min()
    _check_plan(c, m, R, r_idx, budget, res)


def test_invariants_config0_and_config1():
    for idx, nb in ((0, 1), (1, 2)):
        w = workloads.config(idx, nb)
        for b in range(w.B):
            inst = w.instance(b)
            res = oracle.solve(*inst, want_C_last=True, want_bp=True)
            _table_invariants(*inst, res)
            assert res.best_cost < INF


@pytest.mark.parametrize("idx", [2, 3, 4])
def test_invariants_reduced_large_configs(idx):
    """Configurations 2-4 with their value distributions but budgets cut to keep
    the CPU suite short; the last budget of configuration 3 is so small that the
    instance has no admissible plan (a wanted case)."""
    w = workloads.config(idx, 2)
    scale = {2: 6, 3: 8, 4: 16}[idx]
    for b in range(w.B):
        c, m, R, r_idx, budget = w.instance(b)
        budget = budget // scale if b == 0 else int(m.min(axis=1).sum()) - 1 + 2000 * (idx != 3)
        res = oracle.solve(c, m, R, r_idx, budget, want_C_last=True, want_bp=True)
        _table_invariants(c, m, R, r_idx, budget, res)
        if idx == 3 and b == 1:
            assert res.best_cost == INF
        if idx == 4:
            assert res.n_tied > 0                        # injected ties are exercised


def test_smaller_budget_is_a_column_of_the_table():
    w = workloads.config(1, 1)
    c, m, R, r_idx, budget = w.instance(0)
    full = oracle.solve(c, m, R, r_idx, 6000, want_C_last=True, want_bp=True)
    prev = INF
    for e in (0, 500, 2999, 4000, 6000):
        part = oracle.solve(c, m, R, r_idx, e, want_C_last=True, want_bp=True)
        assert (part.C_last == full.C_last[:e + 1]).all()
        assert (part.bp == full.bp[:, :e + 1]).all()
        assert part.best_cost == full.C_last[e].min()
        assert part.best_cost <= prev                    # optimum non-increasing in budget
        prev = part.best_cost
    assert prev < INF
