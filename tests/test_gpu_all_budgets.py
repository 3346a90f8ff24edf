"""GPU parity of the all-budgets outputs: because the table has at-most-e
semantics (optimal substructure, paper section 3.3), one solve answers every
smaller budget.  Checked against the oracle solved separately per budget."""
import numpy as np
import pytest
import torch

import oracle
from paper_2211_13878_amd import binding, workloads

pytestmark = pytest.mark.gpu
INF = binding.GALV_INF


def _solve(w, flags=0):
    sol = binding.Solver(w.B, w.L, w.S, w.E_max, w.nR, flags)
    sol.solve(*binding.upload(w))
    return sol


@pytest.mark.parametrize("S,flags", [(5, 0), (22, 0), (44, 0), (70, 0), (22, binding.GALV_DP_FORCE_INT64),
                                     (22, binding.GALV_DP_FORCE_PACK), (130, binding.GALV_DP_FORCE_PACK | binding.GALV_DP_FORCE_PEEK)])
def test_best_per_budget_matches_oracle_columns(S, flags):
    w = workloads.random_workload(300 + S, 3, 6, S, 900, nR=2, m_range=(0, 200), c_range=(0, 500),
                                  r_range=(0, 200), infeasible=0.1, zero_diagonal=False)
    w.budget[0] = w.E_max
    sol = _solve(w, flags)
    cost, last = (t.cpu().numpy() for t in sol.best_per_budget())
    for b in range(w.B):
        inst = w.instance(b)
        E_b = inst[4]
        ref = oracle.solve(*inst, want_C_last=True)
        want_cost = ref.C_last.min(axis=1)
        want_last = np.where(want_cost < INF, ref.C_last.argmin(axis=1), -1)   # argmin: first minimum
        assert (cost[b, :E_b + 1] == want_cost).all()
        assert (last[b, :E_b + 1] == want_last).all()
        assert (cost[b, E_b + 1:] == INF).all() and (last[b, E_b + 1:] == -1).all()
        assert (cost[b, 1:E_b + 1] <= cost[b, :E_b]).all()          # non-increasing in the budget


@pytest.mark.parametrize("flags", [0, binding.GALV_DP_FORCE_PACK, binding.GALV_DP_FORCE_PACK | binding.GALV_DP_FORCE_PEEK])
def test_backtrack_queries_match_oracle_per_budget(flags):
    w = workloads.random_workload(77, 4, 8, 22, 1500, nR=2, m_range=(0, 250), c_range=(0, 999),
                                  r_range=(0, 300), infeasible=0.1)
    w.budget[:] = [1500, 1200, 700, 1499]
    sol = _solve(w, flags)
    rng = np.random.default_rng(5)
    inst, bud = [], []
    for b in range(w.B):
        E_b = int(w.budget[b])
        for e in [0, E_b, E_b // 2] + list(rng.integers(0, E_b + 1, size=6)):
            inst.append(b); bud.append(int(e))
    # out-of-range queries: beyond the solved budget, negative, bad instance
    inst += [2, 1, 9, -1]; bud += [701, -1, 10, 10]
    qi = torch.tensor(inst, dtype=torch.int32, device="cuda")
    qb = torch.tensor(bud, dtype=torch.int32, device="cuda")
    cost, plan = (t.cpu().numpy() for t in sol.backtrack_queries(qi, qb))
    n_ok = len(inst) - 4
    n_feasible = 0
    for q in range(n_ok):
        c, m, R, r_idx, _ = w.instance(inst[q])
        ref = oracle.solve(c, m, R, r_idx, bud[q])
        assert int(cost[q]) == ref.best_cost, (q, inst[q], bud[q])
        assert (plan[q] == ref.plan).all(), (q, inst[q], bud[q])
        n_feasible += ref.best_cost < INF
    assert 0 < n_feasible < n_ok
    assert (cost[n_ok:] == INF).all() and (plan[n_ok:] == -1).all()


def test_config1_budget_sweep_from_one_solve():
    """One solve of configuration 1 at 16384 units answers the 8 / 12 / 16 thousand-unit budgets."""
    w = workloads.config(1, 2)
    sol = _solve(w)
    budgets = [8192, 12288, 16384, 3000]
    qi = torch.tensor([b for b in range(w.B) for _ in budgets], dtype=torch.int32, device="cuda")
    qb = torch.tensor(budgets * w.B, dtype=torch.int32, device="cuda")
    cost, plan = (t.cpu().numpy() for t in sol.backtrack_queries(qi, qb))
    best, _ = sol.best_per_budget()
    best = best.cpu().numpy()
    for q in range(len(qi)):
        b, e = int(qi[q]), int(qb[q])
        c, m, R, r_idx, _ = w.instance(b)
        ref = oracle.solve(c, m, R, r_idx, e)
        assert int(cost[q]) == ref.best_cost == int(best[b, e])
        assert (plan[q] == ref.plan).all()


def test_call_order_errors():
    w = workloads.random_workload(1, 1, 3, 4, 50, m_range=(0, 9), c_range=(0, 9), r_range=(0, 9))
    sol = binding.Solver(w.B, w.L, w.S, w.E_max, w.nR)
    with pytest.raises(binding.GalvError) as ei:
        sol.best_per_budget()
    assert ei.value.code == binding.GALV_ERR_STATE
    q = torch.zeros(1, dtype=torch.int32, device="cuda")
    with pytest.raises(binding.GalvError) as ei:
        sol.backtrack_queries(q, q)
    assert ei.value.code == binding.GALV_ERR_STATE
