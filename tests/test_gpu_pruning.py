"""Pruning of dominated former strategies in the 32-bit-key sweep.

A former strategy whose cost exceeds a column's minimum by more than the largest transition
cost can neither win nor tie that column's minima; the sweep leaves out rows for which that
holds in every column of a tile.  Results must not depend on it: these cases drive the
pruning to both extremes (nearly everything dropped; nothing dropped, which overflows the
short list of kept rows and takes the fall-back loop) and through mixtures, always against
the oracle with whole tables, and read the library's own statistics to make sure the
intended path ran."""
import numpy as np
import pytest
import torch

from paper_2211_13878_amd import binding, workloads
from test_gpu_parity import check_against_oracle

pytestmark = pytest.mark.gpu


PEEK, NO_PEEK = binding.GALV_DP_FORCE_PEEK, binding.GALV_DP_NO_PEEK
NO_PACK = binding.GALV_DP_NO_PACK          # rolling cost rows + plain back-pointers
WIDE = binding.GALV_DP_FORCE_WIDE_TILES    # 256-column tiles where the variant has such a twin (17 to 256 strategies)
PACK = binding.GALV_DP_FORCE_PACK          # the single packed table (these shapes are too small to choose it)


def reduced_share(w, flags=0):
    sol = binding.Solver(w.B, w.L, w.S, w.E_max, w.nR, flags)
    sol.solve(*binding.upload(w))
    st = sol.stats().cpu().numpy()
    status = sol.status().cpu().numpy()
    sol.close()
    return st, status


@pytest.mark.parametrize("S", [17, 22, 44, 64, 65, 100, 128, 129, 200, 256])
def test_nothing_can_be_pruned(S):
    """Transition costs far above the spread of the layer costs: every row stays alive in every
    tile, more rows than the kept-row list holds (16 up to 64 strategies, 32 beyond), so the
    workgroups take the full loop over all usable rows."""
    w = workloads.random_workload(300 + S, 3, 5, S, 700, nR=2, m_range=(0, 150), c_range=(0, 9),
                                  r_range=(1000, 5000), infeasible=0.05, zero_diagonal=False)
    w.budget[0] = 700
    for flags in (PEEK | PACK, NO_PEEK | PACK, PEEK | NO_PACK, NO_PEEK | NO_PACK, PEEK | PACK | WIDE, NO_PEEK | NO_PACK | WIDE):
        check_against_oracle(w, flags=flags, table_instances=[0, 1, 2], expect_status=binding.GALV_INSTANCE_OK_FAST_U32)
    st, _ = reduced_share(w, PEEK | PACK)
    assert (st[:, 1] > 0).all() and (st[:, 0] >= 0.85 * st[:, 1]).all()     # all but the tiles at the unreachable low budgets
    # the full loop re-reads, through the caches, even the few rows the first fetch had skipped
    assert (st[:, 2] >= 0.85 * st[:, 1]).all() and (st[:, 2] <= st[:, 1]).all()


@pytest.mark.parametrize("S", [8, 22, 44, 128, 200, 256])
def test_nearly_everything_is_pruned(S):
    """Layer costs spread over a range a thousand times the largest transition cost: a handful
    of rows survive per tile."""
    w = workloads.random_workload(400 + S, 3, 6, S, 900, nR=2, m_range=(0, 120), c_range=(0, 100000),
                                  r_range=(0, 90), infeasible=0.05, zero_diagonal=False)
    w.budget[0] = 900
    for flags in (PEEK | PACK, NO_PEEK | PACK, PEEK | NO_PACK, NO_PEEK | NO_PACK, PEEK | PACK | WIDE, NO_PEEK | NO_PACK | WIDE):
        check_against_oracle(w, flags=flags, table_instances=[0, 1, 2], expect_status=binding.GALV_INSTANCE_OK_FAST_U32)
    st, _ = reduced_share(w, NO_PEEK)
    assert (st[:, 2] == st[:, 1]).all()             # every listed row fetched
    st, _ = reduced_share(w, PEEK)
    assert (st[:, 0] < 0.5 * st[:, 1]).all()
    # most rows are not even fetched (instance 0 has the full budget; a tile whose first column is
    # unreachable, as in the small-budget instances, has to fetch every row)
    assert (st[:, 2] >= st[:, 0]).all() and st[0, 2] < 0.8 * st[0, 1]


@pytest.mark.parametrize("seed", range(4))
def test_mixtures_around_the_list_capacity(seed):
    """Transition costs comparable to the cost spread, so that the number of surviving rows
    varies from tile to tile around the capacity of the list (some tiles pruned, some not)."""
    rng = np.random.default_rng(seed)
    S = int(rng.choice([40, 44, 96, 128, 180, 255]))
    spread = int(rng.choice([300, 1000, 3000]))
    w = workloads.random_workload(500 + seed, 3, 6, S, 1200, nR=2, m_range=(0, 200), c_range=(0, spread),
                                  r_range=(0, 400), infeasible=0.08, zero_diagonal=False)
    check_against_oracle(w, flags=PEEK | PACK, table_instances=[0, 1, 2])
    for flags in (NO_PEEK | PACK, PEEK | binding.GALV_DP_BP_U8, PEEK | PACK | binding.GALV_DP_STREAMS(3), PEEK | NO_PACK,
                  NO_PACK | binding.GALV_DP_STREAMS(2), PEEK | PACK | WIDE, WIDE | binding.GALV_DP_BP_U8):
        check_against_oracle(w, flags=flags, table_instances=[1])


def test_statistics_on_a_named_configuration_and_on_other_paths():
    w = workloads.config(1)
    st, status = reduced_share(w, PEEK)
    assert (status == binding.GALV_INSTANCE_OK_FAST_U32).all()
    assert (st[:, 1] > 0).all() and (st[:, 0] < 0.3 * st[:, 1]).all() and (st[:, 2] < 0.6 * st[:, 1]).all()
    st, status = reduced_share(workloads.config(1, 2), binding.GALV_DP_NO_U32)
    assert (status == binding.GALV_INSTANCE_OK_FAST).all() and (st == 0).all()
