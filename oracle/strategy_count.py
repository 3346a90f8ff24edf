"""Plain check of the strategy space of paper section 3.2 — test infrastructure only.

Generate-and-filter (not the product's constructive recursion): list every
sequence of up to three (paradigm, degree) levels with degrees among the powers
of two, and keep those that obey the three tree rules of the section — one level
per paradigm used, no paradigm twice, degrees >= 2 whose product is the group
size — and, optionally, Takeaway #3 (never DP together with SDP).
"""
import itertools


def count_group(group: int, prune_dp_sdp: bool, paradigms=("DP", "SDP", "TP"), ordered: bool = True) -> set:
    degrees = [d for d in (2, 4, 8, 16, 32, 64, 128, 256, 512, 1024) if d <= max(group, 2)]
    kept = set()
    for depth in range(0, 4):
        for names in itertools.product(paradigms, repeat=depth):
            if len(set(names)) != depth:
                continue
            if not ordered and list(names) != sorted(names, key=paradigms.index):
                continue
            if prune_dp_sdp and "DP" in names and "SDP" in names:
                continue
            for degs in itertools.product(degrees, repeat=depth):
                prod = 1
                for d in degs:
                    prod *= d
                if prod == group:
                    kept.add(tuple(zip(names, degs)))
    return kept


def count_all(n_devices: int, prune_dp_sdp: bool) -> int:
    total, pp = 0, 1
    while pp <= n_devices:
        total += len(count_group(n_devices // pp, prune_dp_sdp))
        pp *= 2
    return total
