"""Pins for oracle/coarsen.py — CPU only.  The coarse problem is pinned to what it must mean
for the ORIGINAL problem: its optimum equals a brute force over original plans restricted to
one strategy per fused group under the rounded memory accounting; every coarse plan is a
feasible original plan of the same cost; and the special cases that must be lossless are."""
import itertools

import numpy as np
import pytest

import oracle
from oracle import coarsen as oc
from oracle.bruteforce import brute_force, plan_cost, plan_memory
from paper_2211_13878_amd import workloads

INF = oracle.INF


@pytest.fixture(scope="module", autouse=True)
def _built():
    oracle.build()


def tiny(seed, L=5, S=3, E=60, nR=2):
    return workloads.random_workload(seed, 2, L, S, E, nR=nR, m_range=(0, 25), c_range=(0, 40),
                                     r_range=(0, 15), infeasible=0.1, zero_diagonal=False)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("fuse,gran", [(1, 1), (2, 1), (1, 4), (2, 3), (3, 7), (5, 2), (8, 1)])
def test_coarse_optimum_is_the_restricted_fine_optimum(seed, fuse, gran):
    w = tiny(seed)
    for b in range(w.B):
        c, m, R, r_idx, E = w.instance(b)
        c2, m2, r2, E2 = oc.coarsen(c, m, R, r_idx, E, fuse, gran)
        got = oracle.solve(c2, m2, R, r2, E2)
        # brute force over ORIGINAL plans that are constant on each group
        Lc = -(-w.L // fuse)
        best = None
        for cp in itertools.product(range(w.S), repeat=Lc):
            plan = oc.expand_plan(cp, w.L, fuse)
            if any(m[l, s] > E for l, s in enumerate(plan)):
                continue
            units = 0
            for j in range(Lc):
                grp = range(j * fuse, min(w.L, (j + 1) * fuse))
                units += -(-sum(int(m[l, plan[l]]) for l in grp) // gran)
            if units > E // gran:
                continue
            key = (plan_cost(c, R, r_idx, plan), tuple(reversed(cp)))
            best = key if best is None or key < best else best
        if best is None:
            assert got.best_cost == INF
            continue
        assert got.best_cost == best[0] and tuple(reversed(got.plan.tolist())) == best[1]
        # the expanded plan is feasible for the original problem at the very same cost
        plan = oc.expand_plan(got.plan, w.L, fuse)
        assert plan_memory(m, plan) <= E and plan_cost(c, R, r_idx, plan) == got.best_cost
        # hence an upper bound of the fine optimum
        fine = brute_force(c, m, R, r_idx, E)
        assert fine[0] <= got.best_cost


def test_identity_and_lossless_granularity():
    w = tiny(11, L=6, S=4, E=96)
    for b in range(w.B):
        c, m, R, r_idx, E = w.instance(b)
        c1, m1, r1, E1 = oc.coarsen(c, m, R, r_idx, E, 1, 1)
        usable = m <= E
        assert (c1 == c).all() and (r1 == r_idx).all() and E1 == E and (m1[usable] == m[usable]).all()
        assert (m1[~usable] > E).all()
        # all memories and the budget multiples of g: counting in units of g loses nothing
        g = 8
        mg, Eg = (m // g) * g, (E // g) * g
        fine = oracle.solve(c, mg, R, r_idx, Eg)
        c2, m2, r2, E2 = oc.coarsen(c, mg, R, r_idx, Eg, 1, g)
        coarse = oracle.solve(c2, m2, R, r2, E2)
        assert coarse.best_cost == fine.best_cost and (coarse.plan == fine.plan).all()


def test_fusing_identical_layers_with_free_self_transition_can_only_cost_flexibility():
    # identical layers, R(s,s) = 0: the fused cost of a group is fuse * c(s); hand-checkable case
    S, L = 3, 4
    c = np.tile(np.array([[10, 6, 3]], np.int64), (L, 1))
    m = np.tile(np.array([[1, 2, 4]], np.int32), (L, 1))
    R = np.array([[[0, 5, 5], [5, 0, 5], [5, 5, 0]]], np.int64)
    c2, m2, r2, E2 = oc.coarsen(c, m, R, None, 9, 2, 1)
    assert c2.tolist() == [[20, 12, 6], [20, 12, 6]] and m2.tolist() == [[2, 4, 8], [2, 4, 8]] and E2 == 9
    # fine optimum within 9 units: e.g. (2,1,1,1): memory 4+2+2+2=10 no; (1,1,1,1): 8 -> 24; (2,1,1,0): 9 -> 3+5+6+6+5+10=35
    assert oracle.solve(c, m, R, None, 9).best_cost == 24
    # coarse: groups (1,1): memory 8 -> 24 as well; with budget 10: fine can take (2,1,1,1)=10 -> 3+5+6+6+6=26 no gain
    assert oracle.solve(c2, m2, R, np.zeros(2, np.int32), E2).best_cost == 24
    # inner-boundary transition is charged: R(s,s) = 7 on the diagonal adds 7 per fused pair
    R7 = R + 7 * np.eye(3, dtype=np.int64)[None]
    c3, _, _, _ = oc.coarsen(c, m, R7, None, 9, 2, 1)
    assert c3.tolist() == [[27, 19, 13], [27, 19, 13]]
    # ragged last group: L = 4, fuse = 3 -> groups of 3 and 1
    c4, m4, _, _ = oc.coarsen(c, m, R7, None, 9, 3, 2)
    assert c4.tolist() == [[44, 32, 23], [10, 6, 3]] and m4.tolist() == [[2, 3, 5], [1, 1, 2]]
