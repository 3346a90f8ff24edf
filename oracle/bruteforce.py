"""The plain definition of the plan search, by enumeration.  Test infrastructure only.

Paper section 3.3 (problem formulation and Eq. 1 unrolled): a plan assigns one
strategy to every layer; its time is the sum of the layers' execution times
plus the transformation cost between each pair of neighbouring layers; it is
admissible when its summed memory does not exceed the budget.  The optimum is
the cheapest admissible plan, "infinity" (Out-Of-Memory) when there is none.

Among equally cheap plans this returns the one that is smallest when read
from the last layer to the first, which is what lowest-index tie-breaking in
the layer recurrence produces.  Pure Python: S**L plans, tiny cases only.
"""
from __future__ import annotations

import itertools

INF = 1 << 62


def plan_cost(c, R, r_idx, plan) -> int:
    total = int(c[0][plan[0]])
    for l in range(1, len(plan)):
        k = 0 if r_idx is None else int(r_idx[l])
        total += int(c[l][plan[l]]) + int(R[k][plan[l - 1]][plan[l]])
    return total


def plan_memory(m, plan) -> int:
    return sum(int(m[l][s]) for l, s in enumerate(plan))


def brute_force(c, m, R, r_idx, budget):
    """Return (best_cost, plan) with plan a list of ints, or (INF, [-1]*L)."""
    L, S = len(c), len(c[0])
    if getattr(R, "ndim", 3) == 2:
        R = [R]
    best_key, best_plan = None, None
    for plan in itertools.product(range(S), repeat=L):
        if plan_memory(m, plan) > budget:
            continue
        key = (plan_cost(c, R, r_idx, plan),) + tuple(reversed(plan))
        if best_key is None or key < best_key:
            best_key, best_plan = key, plan
    if best_plan is None:
        return INF, [-1] * L
    return best_key[0], list(best_plan)


def brute_force_cells(c, m, R, r_idx, budget):
    """Every table cell from the plain definition, by enumeration (tiny cases only).

    C[l][e][s] is the cheapest time of layers 0..l over all partial plans
    (p_0, ..., p_l) that end in p_l = s and use at most e memory units; the
    back-pointer of that cell is the lowest former strategy p_{l-1} = s' for which
    a partial plan ending in (s', s) attains that minimum (-1 for layer 0 and for
    cells no partial plan reaches).  Returns (C, bp, n_tied): C and bp as nested
    lists [L][budget+1][S] (the last layer's C is the table whose minimum over s at
    e = budget is the optimum of `brute_force`) and the number of cells of layers
    >= 1 whose minimum is attained by two or more former strategies.
    """
    L, S = len(c), len(c[0])
    if getattr(R, "ndim", 3) == 2:
        R = [R]
    C = [[[INF] * S for _ in range(budget + 1)] for _ in range(L)]
    bp = [[[-1] * S for _ in range(budget + 1)] for _ in range(L)]
    n_tied = 0
    for l in range(L):
        # cheapest partial plan per (memory used, former strategy, last strategy)
        best = {}
        for plan in itertools.product(range(S), repeat=l + 1):
            mem = plan_memory(m, plan)
            if mem > budget:
                continue
            cost = plan_cost(c, R, r_idx, plan)
            key = (mem, plan[-2] if l else -1, plan[-1])
            if key not in best or cost < best[key]:
                best[key] = cost
        for e in range(budget + 1):
            for s in range(S):
                cands = [min((v for (mem, a, b), v in best.items() if a == sp and b == s and mem <= e),
                             default=INF)
                         for sp in ([-1] if l == 0 else range(S))]
                low = min(cands)
                if low < INF:
                    C[l][e][s] = low
                    bp[l][e][s] = -1 if l == 0 else cands.index(low)     # lowest index wins ties
                    n_tied += l > 0 and cands.count(low) > 1
    return C, bp, n_tied
