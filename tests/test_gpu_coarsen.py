"""Coarsening pre-pass on the GPU (galv_dp_coarsen, galv_dp_expand_plan) against oracle/coarsen.py,
array by array, and end to end through the solver."""
import numpy as np
import pytest
import torch

import oracle
from oracle import coarsen as oc
from oracle.bruteforce import plan_cost, plan_memory
from paper_2211_13878_amd import binding, workloads

pytestmark = pytest.mark.gpu
INF = binding.GALV_INF


def _coarsen_gpu(w, fuse, gran, drop_r_idx=False):
    c, m, R, r_idx, budget = binding.upload(w)
    return binding.galv_dp_coarsen(fuse, gran, c, m, R, None if drop_r_idx else r_idx, budget), (R,)


@pytest.mark.parametrize("fuse,gran", [(1, 1), (2, 1), (1, 16), (3, 5), (4, 64), (7, 3), (40, 1000)])
@pytest.mark.parametrize("S,L", [(1, 1), (5, 7), (22, 32), (70, 9)])
def test_arrays_match_oracle(fuse, gran, S, L):
    w = workloads.random_workload(7000 + 31 * S + L, 3, L, S, 5000, nR=2, m_range=(0, 900), c_range=(0, 10**6),
                                  r_range=(0, 10**5), infeasible=0.1, zero_diagonal=False)
    (c2, m2, r2, e2), _ = _coarsen_gpu(w, fuse, gran)
    for b in range(w.B):
        c, m, R, r_idx, E = w.instance(b)
        ec, em, er, eE = oc.coarsen(c, m, R, r_idx, E, fuse, gran)
        assert (c2[b].cpu().numpy() == ec).all() and (m2[b].cpu().numpy() == em).all()
        assert (r2[b].cpu().numpy() == er).all() and int(e2[b]) == eE
    (c3, m3, r3, _), _ = _coarsen_gpu(w, fuse, gran, drop_r_idx=True)
    c, m, R, _, E = w.instance(0)
    ec, em, er, _ = oc.coarsen(c, m, R, None, E, fuse, gran)
    assert (c3[0].cpu().numpy() == ec).all() and (r3[0].cpu().numpy() == 0).all()


@pytest.mark.parametrize("fuse,gran", [(2, 8), (4, 1), (3, 32)])
def test_end_to_end_coarse_solve_and_expanded_plan(fuse, gran):
    w = workloads.config(1)
    (c2, m2, r2, e2), (R,) = _coarsen_gpu(w, fuse, gran)
    Lc = c2.shape[1]
    sol = binding.Solver(w.B, Lc, w.S, w.E_max // gran, w.nR)
    cost, _ = sol.solve(c2, m2, R, r2, e2)
    plan = binding.galv_dp_expand_plan(sol.backtrack(), w.L, fuse).cpu().numpy()
    cost = cost.cpu().numpy()
    fine = oracle.solve_workload(w, threads=8)
    for b in range(w.B):
        c, m, Rb, r_idx, E = w.instance(b)
        ec, em, er, eE = oc.coarsen(c, m, Rb, r_idx, E, fuse, gran)
        ref = oracle.solve(ec, em, Rb, er, eE)
        assert int(cost[b]) == ref.best_cost
        assert plan[b].tolist() == (oc.expand_plan(ref.plan, w.L, fuse) if ref.best_cost < INF else [-1] * w.L)
        if ref.best_cost < INF:
            p = plan[b].tolist()
            assert plan_memory(m, p) <= E and plan_cost(c, Rb, r_idx, p) == cost[b] >= fine[b].best_cost
    sol.close()


def test_invalid_values_stay_invalid_and_argument_errors():
    w = workloads.random_workload(5, 3, 6, 4, 300, m_range=(0, 50), c_range=(0, 100), r_range=(0, 10))
    w.c[0, 2, 1] = -5
    w.m[1, 3, 2] = -1
    (c2, m2, r2, e2), (R,) = _coarsen_gpu(w, 2, 4)
    assert int(c2[0, 1, 1]) == -1 and int(m2[1, 1, 2]) == -1
    sol = binding.Solver(w.B, 3, w.S, 300 // 4, w.nR)
    sol.solve(c2, m2, R, r2, e2)
    assert sol.status().cpu().tolist()[:2] == [binding.GALV_INSTANCE_BAD_VALUE] * 2
    sol.close()
    c, m, R, r_idx, budget = binding.upload(w)
    lib = binding.load_library()
    ptr = lambda t: t.data_ptr()
    for fuse, gran in [(0, 1), (1, 0), (-1, 1)]:
        rc = lib.galv_dp_coarsen(3, 6, 4, 1, fuse, gran, ptr(c), ptr(m), ptr(R), ptr(r_idx), ptr(budget),
                                 ptr(c2), ptr(m2), ptr(r2), ptr(e2), None)
        assert rc == binding.GALV_ERR_INVALID_ARG
    assert lib.galv_dp_expand_plan(3, 6, 0, ptr(r2), ptr(r2), None) == binding.GALV_ERR_INVALID_ARG
