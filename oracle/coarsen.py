"""Coarse-grained exploration (closing remark of the "Dynamic Programming Search" paragraph,
paper section 3.3: fuse several layers, count memory in larger units) — test infrastructure only.

Written as plain loops over one instance.  A fused layer runs one strategy: its time is the
sum of its layers' times plus the same-strategy transition cost at every inner boundary; its
memory is the sum of its layers' memory in units of g, rounded up; the budget is rounded down.
"""
import numpy as np


def coarsen(c, m, R, r_idx, budget, fuse, gran):
    """One instance: c, m [L][S]; R [nR][S][S]; r_idx [L] or None -> (c', m', r_idx', budget')."""
    L, S = c.shape
    Lc = -(-L // fuse)
    Ec = budget // gran
    c2 = np.zeros((Lc, S), np.int64)
    m2 = np.zeros((Lc, S), np.int32)
    r2 = np.zeros(Lc, np.int32)
    for j in range(Lc):
        layers = range(j * fuse, min(L, (j + 1) * fuse))
        r2[j] = 0 if r_idx is None else r_idx[layers[0]]
        for s in range(S):
            cost = sum(int(c[l, s]) for l in layers)
            cost += sum(int(R[0 if r_idx is None else r_idx[l], s, s]) for l in layers[1:])
            mem = sum(int(m[l, s]) for l in layers)
            units = -(-mem // gran)
            fits = all(int(m[l, s]) <= budget for l in layers) and units <= Ec
            c2[j, s] = cost
            m2[j, s] = units if fits else Ec + 1
    return c2, m2, r2, Ec


def expand_plan(coarse_plan, n_layers, fuse):
    return [int(coarse_plan[l // fuse]) for l in range(n_layers)]
