"""Algorithm 1 of the paper (section 3.3, "Optimization Workflow"), plainly — test infrastructure only.

The loop nest as the paper states it: batch sizes in ascending order; for each
pipeline degree P in 1, 2, 4, ..., N the model is cut into P stages of
consecutive layers, as even as the layer count allows (the first L mod P stages
take the extra layer), each stage is searched by the dynamic program of Eq. 1
on its own, the stage optima add up to C_P (transfers between stages are not
charged), C_opt is the smallest C_P, and the answer is the largest B / C_opt
seen before the first batch size for which every degree runs out of memory.
Throughput is held as an exact fraction; the first batch size wins a tie.
"""
from fractions import Fraction

import numpy as np

from .binding import solve
from .strategy_count import count_group

INF = 1 << 62


def pipeline_partition(n_layers: int, pp: int):
    base, extra = divmod(n_layers, pp)
    cuts, lo = [], 0
    for i in range(pp):
        hi = lo + base + (1 if i < extra else 0)
        cuts.append((lo, hi))
        lo = hi
    return cuts


def strategy_counts(n_devices: int, prune_dp_sdp: bool = True) -> dict:
    counts, pp = {}, 1
    while pp <= n_devices:
        counts[pp] = len(count_group(n_devices // pp, prune_dp_sdp))
        pp *= 2
    return counts


def optimize(model, n_devices: int, budget: int, batch_sizes):
    """Returns dict(tpt=Fraction, batch, pp, cost, plans=[per-stage plan], n_explored, c_p=[[...]])."""
    degrees = []
    pp = 1
    while pp <= n_devices:
        degrees.append(pp)
        pp *= 2
    best = dict(tpt=Fraction(0), batch=None, pp=None, cost=None, plans=None, n_explored=0, c_p=[],
                stopped=False)
    for batch in batch_sizes:
        costs, plans = [], []
        for pp in degrees:
            if pp > model.n_layers:           # a stage cannot be empty
                costs.append(INF); plans.append(None)
                continue
            c_p, stage_plans = 0, []
            for lo, hi in pipeline_partition(model.n_layers, pp):
                c, m, R = model.stage_tables(batch, pp, lo, hi)
                r = solve(c, m, R[None], np.zeros(hi - lo, np.int32), budget)
                c_p = INF if (c_p >= INF or r.best_cost >= INF) else c_p + r.best_cost
                stage_plans.append(r.plan.tolist())
            costs.append(c_p); plans.append(stage_plans)
        best["c_p"].append(costs)
        c_opt = min(costs)
        if c_opt >= INF:
            best["stopped"] = True
            return best                        # Out-Of-Memory
        best["n_explored"] += 1
        assert c_opt > 0, "an iteration takes time: throughput B / 0 is not defined"
        tpt = Fraction(batch, c_opt)
        if tpt > best["tpt"]:
            k = costs.index(c_opt)
            best.update(tpt=tpt, batch=batch, pp=degrees[k], cost=c_opt, plans=plans[k])
    return best
