"""The solve and the backtrack only enqueue kernels, events and waits (no allocation, no host
synchronisation, no memset), so a caller may capture them into a HIP graph and replay it.
Each replay is checked against the oracle, with eager work and synchronisations in between and
with the input VALUES changed in place between replays (the graph holds pointers, not data)."""
import pytest
import torch

import oracle
from paper_2211_13878_amd import binding, workloads

pytestmark = pytest.mark.gpu


WIDE_PACKED = binding.GALV_DP_FORCE_PACK | binding.GALV_DP_FORCE_PEEK | binding.GALV_DP_FORCE_WIDE_TILES


@pytest.mark.parametrize("n_streams,extra,S", [(1, 0, 40), (3, 0, 40),
                                               (2, binding.GALV_DP_FORCE_PACK | binding.GALV_DP_FORCE_PEEK, 40),
                                               (2, WIDE_PACKED, 100)])     # 256-column tiles: > 64 KB of LDS per workgroup
def test_capture_and_replay(n_streams, extra, S):
    shapes = dict(B=6, L=10 if S <= 64 else 6, S=S, E_max=1800 if S <= 64 else 900)
    ws = [workloads.random_workload(800 + i, shapes["B"], shapes["L"], shapes["S"], shapes["E_max"], nR=2,
                                    m_range=(0, 250), c_range=(0, 5000), r_range=(0, 900), infeasible=0.06)
          for i in range(4)]
    sol = binding.Solver(shapes["B"], shapes["L"], shapes["S"], shapes["E_max"], 2, binding.GALV_DP_STREAMS(n_streams) | extra)
    dev = [t.clone() for t in binding.upload(ws[0])]
    # eager reference run (also warms up everything the capture must not do for the first time)
    sol.solve(*dev)
    sol.backtrack()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        sol.solve(*dev)
        sol.backtrack()
    for i, w in enumerate(ws):
        for dst, src in zip(dev, binding.upload(w)):
            dst.copy_(src)                                  # new values, same buffers
        torch.cuda.synchronize()
        sol.best_cost.fill_(-7)
        sol.plan.fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        cost, plan = sol.best_cost.cpu().numpy(), sol.plan.cpu().numpy()
        for b, ref in enumerate(oracle.solve_workload(w, threads=4)):
            assert int(cost[b]) == ref.best_cost and (plan[b] == ref.plan).all(), (i, b)
        # eager work between replays
        sol.solve(*dev)
        torch.cuda.synchronize()
        assert (sol.best_cost.cpu().numpy() == cost).all()
    del graph
    sol.close()
