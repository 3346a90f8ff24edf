"""Internal streams (GALV_DP_STREAMS): instances are independent, so spreading their layer
sweeps over several streams must change nothing but timing."""
import pytest
import torch

import oracle
from paper_2211_13878_amd import binding, workloads
from test_gpu_parity import check_against_oracle

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("n_streams", [1, 2, 3, 6, 16])
@pytest.mark.parametrize("B", [1, 5, 7])
def test_parity_with_explicit_stream_counts(n_streams, B):
    w = workloads.random_workload(500 + B, B, 9, 23, 1500, nR=2, m_range=(0, 300), c_range=(0, 60),
                                  r_range=(0, 20), infeasible=0.08, zero_diagonal=False)
    for extra in (0, binding.GALV_DP_FORCE_PACK | binding.GALV_DP_FORCE_PEEK, binding.GALV_DP_FORCE_INT64, binding.GALV_DP_BP_U8):
        check_against_oracle(w, flags=binding.GALV_DP_STREAMS(n_streams) | extra,
                             table_instances=[0, B - 1])


def test_repeated_solves_and_caller_side_stream():
    """Back-to-back solves on one handle with changing inputs, issued on a caller's stream: each
    solve must be ordered after the previous one's sweeps and before the reads that follow."""
    ws = [workloads.random_workload(600 + i, 6, 12, 22, 2000, m_range=(0, 250), c_range=(0, 1000),
                                    r_range=(0, 300), infeasible=0.05) for i in range(3)]
    sol = binding.Solver(6, 12, 22, 2000, 1, binding.GALV_DP_STREAMS(3) | binding.GALV_DP_FORCE_PACK)
    side = torch.cuda.Stream()
    results = []
    devs = [binding.upload(w) for w in ws]
    torch.cuda.synchronize()
    with torch.cuda.stream(side):
        for dev in devs:
            cost, _ = sol.solve(*dev)
            plan = sol.backtrack()
            results.append((cost.clone(), plan.clone()))
    side.synchronize()
    for w, (cost, plan) in zip(ws, results):
        for b, ref in enumerate(oracle.solve_workload(w, threads=4)):
            assert int(cost[b]) == ref.best_cost and (plan[b].cpu().numpy() == ref.plan).all()
    sol.close()


def test_too_many_streams_is_an_error():
    with pytest.raises(binding.GalvError) as e:
        binding.galv_dp_workspace_bytes(binding.make_desc(4, 4, 6, 256, flags=binding.GALV_DP_STREAMS(17)))
    assert e.value.code == binding.GALV_ERR_INVALID_ARG


def test_automatic_stream_count_follows_the_budgets_the_last_solve_met():
    """With no stream count asked for, a solve sizes its launches by the budget tiles the solve
    before it found (the budgets live on the device; before any solve the largest possible count
    stands in).  Whatever it picks, the results are the oracle's."""
    import dataclasses
    import numpy as np
    B, L, S, E = 32, 3, 44, 16383
    big = workloads.random_workload(910, B, L, S, E, m_range=(0, 2500), c_range=(0, 10 ** 5),
                                    r_range=(0, 3 * 10 ** 4), infeasible=0.05)
    big = dataclasses.replace(big, budget=np.full_like(big.budget, E))
    small = dataclasses.replace(big, budget=np.full_like(big.budget, 1500))
    sol = binding.Solver(B, L, S, E, 1, 0)
    before = sol.config()["streams"]
    assert before >= 2                      # a launch of this shape is worth splitting
    used = []
    for w in (big, small, small, big):
        dev = binding.upload(w)
        cost, _ = sol.solve(*dev)
        plan = sol.backtrack()
        cost, plan = cost.cpu().numpy(), plan.cpu().numpy()      # (waits for the solve)
        used.append(sol.config()["streams"])
        for b, ref in enumerate(oracle.solve_workload(w, threads=8)):
            assert int(cost[b]) == ref.best_cost and (plan[b] == ref.plan).all(), (w is big, b)
    sol.close()
    # first solve: nothing seen yet; second: what the first met (the large budgets); third: the
    # small budgets, a sixth of the columns, one launch per layer; fourth: still the small ones
    assert used[0] == before and used[1] == before and used[2] == 1 and used[3] == 1, used
