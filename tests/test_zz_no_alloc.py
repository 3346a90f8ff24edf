"""galv_dp_solve_static — the entry point that allocates nothing — against the handle-based
entry points (galv_dp_create + galv_dp_solve_batched + galv_dp_backtrack) on the same inputs.
Both run the same kernels, one over the caller's workspace, the other over the fixed array
inside the library; costs, last strategies and plans must be equal bit for bit, also on a
second, smaller call that finds the first call's contents in the array."""
import pytest
import torch

from paper_2211_13878_amd import binding, workloads

pytestmark = pytest.mark.gpu


def via_handle(w, flags=0):
    sol = binding.Solver(w.B, w.L, w.S, w.E_max, w.nR, flags | binding.GALV_DP_STREAMS(1))
    cost, last = sol.solve(*binding.upload(w))
    plan = sol.backtrack()
    torch.cuda.synchronize()
    out = cost.clone(), last.clone(), plan.clone()
    sol.close()
    return out


def via_static(w, flags=0):
    dev = binding.upload(w)
    cost = torch.full((w.B,), -7, dtype=torch.int64, device="cuda")
    last = torch.full((w.B,), -7, dtype=torch.int32, device="cuda")
    plan = torch.full((w.B, w.L), -7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated(), torch.cuda.memory_reserved()
    binding.galv_dp_solve_static(binding.make_desc(w.B, w.L, w.S, w.E_max, w.nR, flags), *dev, cost, last, plan)
    torch.cuda.synchronize()
    assert (torch.cuda.memory_allocated(), torch.cuda.memory_reserved()) == before
    return cost, last, plan


def same(a, b):
    return all(torch.equal(x, y) for x, y in zip(a, b))


def test_two_calls_in_a_row_second_smaller_then_a_wide_one():
    big = workloads.random_workload(501, 3, 6, 22, 1500, nR=2, m_range=(0, 300), c_range=(0, 5000),
                                    r_range=(0, 900), infeasible=0.1, zero_diagonal=False)
    small = workloads.random_workload(502, 2, 4, 6, 300, m_range=(0, 60), c_range=(0, 50),
                                      r_range=(0, 20), infeasible=0.1)
    small.budget[1] = 17                      # ragged, and most likely infeasible
    wide = workloads.random_workload(503, 2, 4, 128, 600, nR=2, m_range=(0, 150), c_range=(0, 99),
                                     r_range=(0, 30), infeasible=0.05)      # > 64 KB of LDS per workgroup
    for w in (big, small, wide, small):
        ref = via_handle(w)
        assert (ref[0] < binding.GALV_INF).any()
        assert same(via_static(w), ref), w.name
    # the other arithmetic paths and the one-byte back-pointers share the array too
    for flags in (binding.GALV_DP_FORCE_INT64, binding.GALV_DP_NO_U32, binding.GALV_DP_BP_U8,
                  binding.GALV_DP_FORCE_PACK | binding.GALV_DP_FORCE_PEEK):
        assert same(via_static(big, flags), via_handle(big, flags))
    assert same(via_static(small), via_handle(small))


def test_matches_the_oracle_on_config0():
    import oracle
    w = workloads.config(0)
    cost, last, plan = via_static(w)
    ref = oracle.solve(*w.instance(0))
    assert int(cost[0]) == ref.best_cost == 33968 and int(last[0]) == ref.best_last
    assert (plan[0].cpu().numpy() == ref.plan).all()


def test_refuses_what_does_not_fit_or_needs_streams():
    w = workloads.random_workload(504, 1, 3, 4, 50, m_range=(0, 9), c_range=(0, 9), r_range=(0, 9))
    dev = binding.upload(w)
    cost = torch.zeros(1, dtype=torch.int64, device="cuda")
    last = torch.zeros(1, dtype=torch.int32, device="cuda")
    plan = torch.zeros((1, 3), dtype=torch.int32, device="cuda")
    too_big = binding.make_desc(8, 32, 22, 16384)
    assert binding.galv_dp_workspace_bytes(too_big) > binding.GALV_DP_STATIC_BYTES
    with pytest.raises(binding.GalvError) as ei:
        binding.galv_dp_solve_static(too_big, *dev, cost, last, plan)
    assert ei.value.code == binding.GALV_ERR_WORKSPACE and "bytes" in str(ei.value)
    with pytest.raises(binding.GalvError) as ei:
        binding.galv_dp_solve_static(binding.make_desc(1, 3, 4, 50, 1, binding.GALV_DP_STREAMS(2)),
                                     *dev, cost, last, plan)
    assert ei.value.code == binding.GALV_ERR_INVALID_ARG
    with pytest.raises(binding.GalvError) as ei:
        binding.galv_dp_solve_static(binding.make_desc(1, 3, 4, 50), *dev, cost, last, None)
    assert ei.value.code == binding.GALV_ERR_INVALID_ARG
