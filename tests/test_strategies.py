"""Decision-tree strategy enumerator (paper section 3.2) against the paper's
printed counts and an independent generate-and-filter count."""
import os

import pytest

from oracle.strategy_count import count_all, count_group
from paper_2211_13878_amd.strategies import enumerate_strategies, group_strategies

GOLD = {ln.split()[0]: int(ln.split()[1])
        for ln in open(os.path.join(os.path.dirname(__file__), "golden", "strategy_counts.txt"))
        if not ln.startswith("#")}


def test_paper_counts_on_8_gpus():
    assert len(enumerate_strategies(8, prune_dp_sdp=False)) == GOLD["all_8gpu"] == count_all(8, False)
    assert len(enumerate_strategies(8, prune_dp_sdp=True)) == GOLD["pruned_8gpu"] == count_all(8, True)


@pytest.mark.parametrize("n", [1, 2, 4, 8, 16, 64])
@pytest.mark.parametrize("prune", [False, True])
def test_matches_generate_and_filter(n, prune):
    assert set(group_strategies(n, prune)) == count_group(n, prune)
    assert len(enumerate_strategies(n, prune)) == count_all(n, prune)


def test_rules_and_labels():
    strategies = enumerate_strategies(8)
    assert len({s.label for s in strategies}) == len(strategies)
    for s in strategies:
        names = [p for p, _ in s.levels]
        prod = 1
        for _, d in s.levels:
            assert d >= 2 and d & (d - 1) == 0
            prod *= d
        assert len(set(names)) == len(names) and prod * s.pp == 8
        assert not ("DP" in names and "SDP" in names)
    # order matters: 2-DP x 4-TP and 4-TP x 2-DP are distinct candidates
    labels = {s.label for s in strategies}
    assert "2-DP x 4-TP" in labels and "4-TP x 2-DP" in labels and "8-PP / 1" in labels
    # sizes of the sets the dynamic program sees per pipeline degree on 8 GPUs
    assert [len(group_strategies(g)) for g in (8, 4, 2, 1)] == [11, 7, 3, 1]


def test_bad_sizes():
    with pytest.raises(ValueError):
        enumerate_strategies(6)


def test_limited_search_spaces_of_the_comparison():
    dp_tp = enumerate_strategies(8, paradigms=("DP", "TP"), ordered=False, pipeline=False)
    assert len(dp_tp) == GOLD["dp_tp_8gpu"] == len(count_group(8, True, ("DP", "TP"), ordered=False))
    assert {s.label for s in dp_tp} == {"8-DP", "8-TP", "2-DP x 4-TP", "4-DP x 2-TP"}
    dp_pp = enumerate_strategies(8, paradigms=("DP",))
    assert len(dp_pp) == GOLD["dp_pp_8gpu"]
    assert {s.label for s in dp_pp} == {"8-DP", "2-PP / 4-DP", "4-PP / 2-DP", "8-PP / 1"}
    # with the order of the levels counted, DP+TP alone has 6
    assert len(enumerate_strategies(8, paradigms=("DP", "TP"), pipeline=False)) == 6
