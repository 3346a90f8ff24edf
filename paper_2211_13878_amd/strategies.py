"""Candidate hybrid-parallel strategies of one layer (paper section 3.2).

After pipeline parallelism of degree P has split N devices into groups of
G = N / P, a layer's strategy is a decision tree over the paradigms DP
(data), SDP (sharded data) and TP (tensor): one tree level per paradigm used,
no paradigm on two levels, every level's degree a power of two >= 2, the
degrees multiplying to G; the ORDER of the levels matters (it decides which
paradigm gets the faster links).  Takeaway #3 of the same section drops every
tree that mixes DP with SDP.  For N = 8 the paper counts 34 candidates, 22
after Takeaway #3.

This is host-side combinatorics: to the dynamic program a strategy is only an
index s in [0, S); this module supplies S and human-readable labels for plans.
"""
from __future__ import annotations

from dataclasses import dataclass

PARADIGMS = ("DP", "SDP", "TP")


@dataclass(frozen=True)
class Strategy:
    pp: int                               # pipeline degree P
    levels: tuple                         # ((paradigm, degree), ...) from the root down

    @property
    def label(self) -> str:
        inner = " x ".join(f"{d}-{p}" for p, d in self.levels) or "1"
        return f"{self.pp}-PP / {inner}" if self.pp > 1 else inner


def _is_pow2(x: int) -> bool:
    return x >= 1 and (x & (x - 1)) == 0


def group_strategies(group: int, prune_dp_sdp: bool = True, paradigms=PARADIGMS, ordered: bool = True):
    """(paradigm, degree) sequences for a group of `group` devices.

    `paradigms` restricts the tree to a subset (the limited search spaces the paper
    compares against, e.g. DP+TP); `ordered=False` counts a set of levels once, in
    the order of `paradigms`, as those systems do.
    """
    if not _is_pow2(group):
        raise ValueError("group size must be a power of two")
    if not set(paradigms) <= set(PARADIGMS):
        raise ValueError("unknown paradigm")
    out = []

    def grow(prefix, used, remaining):
        if remaining == 1:
            out.append(tuple(prefix))
            return
        for p in paradigms:
            if p in used:
                continue
            if not ordered and prefix and paradigms.index(p) < paradigms.index(prefix[-1][0]):
                continue
            if prune_dp_sdp and ((p == "DP" and "SDP" in used) or (p == "SDP" and "DP" in used)):
                continue
            d = 2
            while d <= remaining:
                if remaining % d == 0:
                    grow(prefix + [(p, d)], used | {p}, remaining // d)
                d *= 2

    grow([], frozenset(), group)
    return out


def enumerate_strategies(n_devices: int, prune_dp_sdp: bool = True, paradigms=PARADIGMS,
                         ordered: bool = True, pipeline: bool = True):
    """All candidates of one layer on `n_devices`, over PP degrees 1, 2, 4, ..., N (only 1 if not `pipeline`)."""
    if not _is_pow2(n_devices):
        raise ValueError("device count must be a power of two")
    result = []
    pp = 1
    while pp <= (n_devices if pipeline else 1):
        for levels in group_strategies(n_devices // pp, prune_dp_sdp, tuple(paradigms), ordered):
            result.append(Strategy(pp, levels))
        pp *= 2
    return result
