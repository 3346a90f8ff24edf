"""Seeded random sweep over shapes, value ranges and flags: costs, plans and (where small enough)
whole tables against the oracle.  Shapes sit on both sides of every kernel variant's limits
(strategies 8 / 16 / 22 / 32 / 44 / 64 / 128, budget tiles of 128 and 256 columns) and value ranges
on both sides of every arithmetic path's limits."""
import numpy as np
import pytest
import torch

import oracle
from paper_2211_13878_amd import binding, workloads

pytestmark = pytest.mark.gpu

FLAGS = [0, binding.GALV_DP_NO_U32, binding.GALV_DP_FORCE_INT64, binding.GALV_DP_BP_U8,
         binding.GALV_DP_BP_U8 | binding.GALV_DP_NO_U32, binding.GALV_DP_STREAMS(3),
         binding.GALV_DP_STREAMS(3) | binding.GALV_DP_BP_U8,
         binding.GALV_DP_FORCE_PEEK, binding.GALV_DP_FORCE_PEEK | binding.GALV_DP_BP_U8 | binding.GALV_DP_STREAMS(2),
         binding.GALV_DP_FORCE_PACK, binding.GALV_DP_FORCE_PACK | binding.GALV_DP_FORCE_PEEK | binding.GALV_DP_STREAMS(2),
         binding.GALV_DP_FORCE_WIDE_TILES | binding.GALV_DP_FORCE_PACK | binding.GALV_DP_FORCE_PEEK,
         binding.GALV_DP_FORCE_WIDE_TILES]


@pytest.mark.parametrize("seed", [11, 12, 13])
def test_random_sweep(seed):
    rng = np.random.default_rng(seed)
    paths = set()
    for it in range(60):
        S = int(rng.choice([1, 2, 3, 7, 8, 9, 11, 12, 16, 17, 18, 21, 22, 23, 31, 32, 33, 34, 40, 43, 44, 45, 63, 64, 65,
                            100, 127, 128, 129, 140]))
        L = int(rng.integers(1, 9))
        B = int(rng.integers(1, 5))
        E = int(rng.choice([0, 1, 63, 64, 127, 128, 129, 255, 256, 257, 500, 1023, 1024, 1025, 2000]))
        if S > 64:
            E = min(E, 600)
        mr = int(rng.choice([0, 1, 5, 50, 400]))
        cr = int(rng.choice([0, 1, 9, 1000, 10**6, 10**8, 10**11]))
        rr = int(rng.choice([0, 1, 9, 1000, 10**6, 2**27 - 1, 2**27, 2**29]))
        w = workloads.random_workload(int(rng.integers(1 << 30)), B, L, S, E, nR=int(rng.integers(1, 4)),
                                      m_range=(0, mr), c_range=(0, cr), r_range=(0, rr),
                                      infeasible=float(rng.choice([0, 0.1, 0.5, 0.95])),
                                      zero_diagonal=bool(rng.integers(2)))
        refs = oracle.solve_workload(w, threads=4)
        full = ([oracle.solve(*w.instance(b), want_C_last=True, want_bp=True) for b in range(w.B)]
                if S * E * L < 400000 else None)
        dev = binding.upload(w)
        for fl in FLAGS:
            sol = binding.Solver(w.B, w.L, w.S, w.E_max, w.nR, fl)
            cost, last = sol.solve(*dev)
            plan = sol.backtrack()
            cost, last, plan = cost.cpu().numpy(), last.cpu().numpy(), plan.cpu().numpy()
            paths.update(int(x) for x in sol.status().cpu().numpy())
            for b, r in enumerate(refs):
                assert int(cost[b]) == r.best_cost and int(last[b]) == r.best_last, (it, S, L, E, fl, b)
                assert (plan[b] == r.plan).all(), (it, S, L, E, fl, b)
            if full is not None:
                for b in range(w.B):
                    C, bp = sol.export_tables(b)
                    Eb = int(w.budget[b])
                    assert (C.cpu().numpy()[:Eb + 1] == full[b].C_last).all(), (it, S, L, E, fl, b)
                    assert (bp.cpu().numpy()[:, :Eb + 1] == full[b].bp).all(), (it, S, L, E, fl, b)
            sol.close()
    assert paths >= {0, 1, 2, 3, 4}          # every arithmetic path was taken somewhere in the sweep
