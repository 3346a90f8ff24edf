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
