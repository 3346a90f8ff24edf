"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, bit
for bit, on the same seeded inputs.  Costs are int64, plans and back-pointers
int32; every comparison is exact equality."""
import os

import numpy as np
import pytest
import torch

import oracle
from oracle.bruteforce import plan_cost, plan_memory
from paper_2211_13878_amd import binding, workloads

pytestmark = pytest.mark.gpu
INF = binding.GALV_INF
assert INF == oracle.INF
# the three arithmetic paths a small-valued instance can be sent down: 32-bit integer keys
# (default), 64-bit keys in 32-bit cells, general 64-bit integers
# single packed table (forced: small shapes would not choose it), cost rows with 32-bit keys, 64-bit keys, int64
ALL_PATHS = (binding.GALV_DP_FORCE_PACK, binding.GALV_DP_NO_PACK, binding.GALV_DP_NO_U32, binding.GALV_DP_FORCE_INT64)
THREADS = max(1, min(16, os.cpu_count() or 1))      # oracle instances solved side by side


def gpu_solve(w, flags=0, tables=(), want_bp=True, clast=()):
    """Run the library on a workload; returns numpy results and exported tables
    (`tables`: C_last and, with want_bp, back-pointers; `clast`: C_last only)."""
    sol = binding.Solver(w.B, w.L, w.S, w.E_max, w.nR, flags)
    dev = binding.upload(w)
    cost, last = sol.solve(*dev)
    plan = sol.backtrack()
    status = sol.status()
    exported = {}
    for b in clast:
        exported[b] = (sol.export_tables(b, False)[0].cpu().numpy(), None)
    for b in tables:
        C_last, bp = sol.export_tables(b, want_bp)
        exported[b] = (C_last.cpu().numpy(), None if bp is None else bp.cpu().numpy())
    torch.cuda.synchronize()
    out = (cost.cpu().numpy(), last.cpu().numpy(), plan.cpu().numpy(), status.cpu().numpy(), exported)
    sol.close()
    return out


def oracle_refs(w, ids, table_instances=(), clast_instances=(), threads=4):
    """Oracle results per instance id: full tables for `table_instances`, the last layer's
    cost table for `clast_instances`, optimum and plan for the rest."""
    ids = list(ids)
    tab, cl = set(table_instances), set(clast_instances) - set(table_instances)
    refs = {}
    plain = [b for b in ids if b not in tab and b not in cl]
    refs.update(zip(plain, oracle.solve_workload(w, plain, threads=threads)))
    refs.update(zip(sorted(cl), oracle.solve_workload(w, sorted(cl), threads=threads, want_C_last=True)))
    refs.update(zip(sorted(tab), oracle.solve_workload(w, sorted(tab), threads=threads, want_C_last=True,
                                                      want_bp=True)))
    return refs


def check_against_oracle(w, flags=0, table_instances=(), oracle_instances=None, threads=4,
                         expect_status=None, clast_instances=(), refs=None, allow_vacuous=False):
    """Optimum, last strategy and plan of every instance (or of `oracle_instances`) against the
    oracle; whole exported tables for `table_instances` (C_last and back-pointers) and
    `clast_instances` (C_last).  A table comparison in which no compared cell is finite proves
    nothing (infinity == infinity), so it fails unless the caller says that is intended."""
    cost, last, plan, status, exported = gpu_solve(w, flags, table_instances, clast=clast_instances)
    ids = list(range(w.B) if oracle_instances is None else oracle_instances)
    if refs is None:
        refs = oracle_refs(w, sorted(set(ids) | set(table_instances) | set(clast_instances)),
                           table_instances, clast_instances, threads)
    for b in ids:
        ref = refs[b]
        assert int(cost[b]) == ref.best_cost, (w.name, b)
        assert int(last[b]) == ref.best_last, (w.name, b)
        assert (plan[b] == ref.plan).all(), (w.name, b)
    if expect_status is not None:
        assert (status == expect_status).all(), status
    finite_cells = reachable_bp = 0
    for b in sorted(set(table_instances) | set(clast_instances)):
        ref = refs[b]
        C_last, bp = exported[b]
        E_b = int(w.budget[b])
        assert (C_last[:E_b + 1] == ref.C_last).all(), (w.name, b)
        assert (C_last[E_b + 1:] == INF).all()
        finite_cells += int((ref.C_last < INF).sum())
        if b in table_instances:
            assert (bp[:, :E_b + 1] == ref.bp).all(), (w.name, b)
            assert (bp[:, E_b + 1:] == -1).all()
            reachable_bp += int((ref.bp[-1] >= 0).sum())
    if (table_instances or clast_instances) and not allow_vacuous:
        assert finite_cells > 0, "every compared cost cell is infinite: the comparison shows nothing"
        if table_instances and w.L > 1:
            assert reachable_bp > 0, "no reachable back-pointer in the last layer"
    return cost, last, plan, status


def check_properties(w, cost, last, plan):
    """Checks that hold at any size: the plan re-evaluates to the reported cost and fits."""
    for b in range(w.B):
        c, m, R, r_idx, budget = w.instance(b)
        if cost[b] == INF:
            assert last[b] == -1 and (plan[b] == -1).all()
            continue
        p = [int(s) for s in plan[b]]
        assert all(0 <= s < w.S for s in p) and p[-1] == last[b]
        assert plan_cost(c, R, r_idx, p) == cost[b]
        assert plan_memory(m, p) <= budget


# ------------------------------------------------------------- named configs

def test_config0_tables_and_golden():
    w = workloads.config(0)
    cost, last, plan, status = check_against_oracle(w, table_instances=[0],
                                                    expect_status=binding.GALV_INSTANCE_OK_FAST_U32)
    assert int(cost[0]) == 33968 and list(plan[0]) == [3, 4, 0, 0]   # tests/golden
    check_against_oracle(w, flags=binding.GALV_DP_NO_U32, table_instances=[0],
                         expect_status=binding.GALV_INSTANCE_OK_FAST)
    check_against_oracle(w, flags=binding.GALV_DP_FORCE_INT64, table_instances=[0],
                         expect_status=binding.GALV_INSTANCE_OK_INT64)


def test_config1_full_batch_with_tables():
    w = workloads.config(1)
    cost, last, plan, _ = check_against_oracle(w, table_instances=[0, 5], threads=8,
                                               expect_status=binding.GALV_INSTANCE_OK_FAST_U32)
    check_properties(w, cost, last, plan)
    assert (cost < INF).all()
    check_against_oracle(w, flags=binding.GALV_DP_NO_U32, table_instances=[3], threads=8,
                         expect_status=binding.GALV_INSTANCE_OK_FAST)


def test_config1_int64_path_prefix():
    w = workloads.config(1, 2)
    check_against_oracle(w, flags=binding.GALV_DP_FORCE_INT64, table_instances=[1],
                         expect_status=binding.GALV_INSTANCE_OK_INT64)


def test_config2_full_batch():
    """Every instance against the oracle: optimum, plan and the whole last-layer cost table;
    all back-pointers for two of them."""
    w = workloads.config(2)
    cost, last, plan, _ = check_against_oracle(w, table_instances=[3, 28], clast_instances=range(w.B),
                                               threads=THREADS,
                                               expect_status=binding.GALV_INSTANCE_OK_FAST_U32)
    check_properties(w, cost, last, plan)


def test_config3_full_size_every_instance():
    """Whole batch on the GPU in the benchmark's launch configuration; the oracle re-solves
    every instance (one of them, number 30, has no plan: its cheapest memory exceeds its
    budget): optimum, plan and the whole last-layer cost table for all 64, every back-pointer
    for two."""
    w = workloads.config(3)
    cost, last, plan, _ = check_against_oracle(w, table_instances=[21, 63], clast_instances=range(w.B),
                                               threads=THREADS,
                                               expect_status=binding.GALV_INSTANCE_OK_FAST_U32)
    check_properties(w, cost, last, plan)
    assert list(np.flatnonzero(cost == INF)) == [30]


# ---- configuration 4 at full size (16 x 1.4e11 candidates: two minutes of oracle per instance)

def torch_checksum(t, chunk_rows=None):
    """oracle/checksum.py's table checksum, retyped for a device tensor (int64 wraps like uint64)."""
    flat = t.reshape(-1)
    total = torch.zeros((), dtype=torch.int64, device=t.device)
    step = 1 << 26
    for lo in range(0, flat.numel(), step):
        x = flat[lo:lo + step].to(torch.int64) + 3
        i = torch.arange(lo, lo + x.numel(), dtype=torch.int64, device=t.device)
        wgt = (i * -7046029254386353131 + 0x7F4A7C15) | 1          # 0x9E3779B97F4A7C15 as int64
        total = total + (x * wgt).sum()
    return int(total.item()) & 0xFFFFFFFFFFFFFFFF


def read_config4_golden():
    rows = {}
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "config4_full_budget.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            v = [int(x) for x in line.split()]
            rows[v[0]] = dict(cost=v[1], last=v[2], n_tied=v[3], sum_C=v[4], sum_bp=v[5], plan=v[6:])
    return rows


@pytest.mark.timeout(900)
def test_config4_full_size_against_stored_oracle_results_and_two_live_instances():
    """Stress shape at full size, in the benchmark's launch configuration.
    (i) All 16 instances against the oracle's stored full-budget results (written by
    tests/golden/make_golden.py from oracle/ only): optimum, last strategy, plan, and the
    checksums of the whole last-layer cost table and of the whole back-pointer table
    (lowest-index ties: the stored tie counts are positive).
    (ii) Two instances are re-solved by the oracle here, at the full budget, and compared cell by
    cell: last-layer costs and every back-pointer."""
    w = workloads.config(4)
    golden = read_config4_golden()
    assert sorted(golden) == list(range(w.B)) and all(g["n_tied"] > 0 for g in golden.values())
    sol = binding.Solver(w.B, w.L, w.S, w.E_max, w.nR)
    cost, last = sol.solve(*binding.upload(w))
    plan = sol.backtrack()
    status = sol.status().cpu().numpy()
    cost, last, plan = cost.cpu().numpy(), last.cpu().numpy(), plan.cpu().numpy()
    assert (status == binding.GALV_INSTANCE_OK_FAST_U32).all() and (cost < INF).all()
    check_properties(w, cost, last, plan)
    live = (5, 12)
    from concurrent.futures import ThreadPoolExecutor
    with ThreadPoolExecutor(max_workers=2) as ex:      # the oracle runs while the GPU side is checked
        futures = {b: ex.submit(oracle.solve, *w.instance(b), want_C_last=True, want_bp=True) for b in live}
        for b in range(w.B):
            g = golden[b]
            assert int(cost[b]) == g["cost"] and int(last[b]) == g["last"], b
            assert list(plan[b]) == g["plan"], b
            C_last, bp = sol.export_tables(b, True)
            finite = int((C_last < INF).sum())
            assert finite > 0.8 * C_last.numel()       # nearly every budget column is reachable here
            assert torch_checksum(C_last) == g["sum_C"], b
            assert torch_checksum(bp) == g["sum_bp"], b
            best = C_last.min(dim=1).values
            assert bool((best[1:] <= best[:-1]).all()) and int(best[-1]) == cost[b]
            if b in live:
                ref = futures[b].result()
                assert ref.best_cost == g["cost"] and list(ref.plan) == g["plan"] and ref.n_tied == g["n_tied"]
                assert torch.equal(C_last.cpu(), torch.from_numpy(ref.C_last)), b
                assert int((ref.C_last < INF).sum()) == finite
                for l in range(w.L):                   # 34 MB of back-pointers per layer
                    assert torch.equal(bp[l].cpu(), torch.from_numpy(ref.bp[l])), (b, l)
                assert int((ref.bp[-1] >= 0).sum()) > 0
                del ref
            del C_last, bp
    sol.close()


def test_config4_full_size_truncated_budget_queries():
    """At-most-e semantics at full size: rows e <= E' of the full-size table, and the plan that
    galv_dp_backtrack_queries returns for (instance, E'), equal an oracle solve at budget E' —
    with E' well above the instances' smallest possible memory, so that the compared cells are
    finite."""
    w = workloads.config(4)
    E_small = 16384
    ids = (3, 14)
    sol = binding.Solver(w.B, w.L, w.S, w.E_max, w.nR)
    sol.solve(*binding.upload(w))
    q_inst = torch.tensor(ids, dtype=torch.int32, device="cuda")
    q_bud = torch.full((len(ids),), E_small, dtype=torch.int32, device="cuda")
    q_cost, q_plan = sol.backtrack_queries(q_inst, q_bud)
    q_cost, q_plan = q_cost.cpu().numpy(), q_plan.cpu().numpy()
    refs = oracle.solve_workload(_with_budget(w, E_small), ids, threads=2, want_C_last=True)
    for q, (b, ref) in enumerate(zip(ids, refs)):
        C_last = sol.export_tables(b, False)[0].cpu().numpy()
        assert ref.best_cost < INF and int((ref.C_last < INF).sum()) > 0.25 * ref.C_last.size
        assert (C_last[:E_small + 1] == ref.C_last).all(), b
        assert q_cost[q] == ref.best_cost and (q_plan[q] == ref.plan).all(), b
    sol.close()


def _with_budget(w, budget):
    import copy
    w2 = copy.copy(w)
    w2.budget = np.full_like(w.budget, budget)
    return w2


_CONFIG4_SMALL = {}


def config4_small_budget():
    """Two instances of the stress shape (S = 128, L = 128, injected ties) with budgets just
    above their smallest possible memory (6617 and 6132 units), so that the oracle can produce
    every cell including back-pointers in seconds and a good part of the cells is finite.
    Returns the workload and the oracle's tables (computed once per session)."""
    if not _CONFIG4_SMALL:
        w = workloads.config(4, 2)
        w.budget[:] = [8000, 9000]
        w.E_max = 9000
        min_mem = w.m.astype(np.int64).min(axis=2).sum(axis=1)
        assert (min_mem < w.budget).all() and (min_mem > 6000).all()
        _CONFIG4_SMALL["w"] = w
        _CONFIG4_SMALL["refs"] = oracle_refs(w, [0, 1], table_instances=[0, 1], threads=2)
        assert all(r.n_tied > 0 and r.best_cost < INF for r in _CONFIG4_SMALL["refs"].values())
    return _CONFIG4_SMALL["w"], _CONFIG4_SMALL["refs"]


def test_config4_shape_small_budget_full_tables():
    """S = 128, L = 128 with injected ties: every cell including back-pointers (lowest-index
    tie-break), on every arithmetic path."""
    w, refs = config4_small_budget()
    for flags in ALL_PATHS:
        check_against_oracle(w, flags=flags, table_instances=[0, 1], refs=refs)


# ------------------------------------------------------- random shapes / edges

@pytest.mark.parametrize("S", [1, 2, 5, 8, 9, 16, 22, 23, 32, 33, 37, 40, 44, 45, 64, 65, 70, 128, 130, 200, 256, 257])
def test_random_shapes_ragged_tiles(S):
    """Several budget tiles with a ragged tail, strategies around every kernel
    variant's group size, narrow values (many ties), m = 0, random budgets,
    infeasible cells, two transition matrices; both arithmetic paths."""
    L = 5 if S > 64 else 7
    E_max = 1337 if S <= 64 else 700
    w = workloads.random_workload(40 + S, 3, L, S, E_max, nR=2, m_range=(0, 300),
                                  c_range=(0, 50), r_range=(0, 20), infeasible=0.08,
                                  zero_diagonal=False)
    w.budget[0] = E_max
    WIDE = binding.GALV_DP_FORCE_WIDE_TILES        # 256-column tiles (the variants for 17 to 256 strategies have such a twin)
    for flags in ALL_PATHS + (binding.GALV_DP_FORCE_PEEK, binding.GALV_DP_FORCE_PEEK | binding.GALV_DP_FORCE_PACK,
                              WIDE | binding.GALV_DP_FORCE_PACK, WIDE | binding.GALV_DP_FORCE_PEEK | binding.GALV_DP_FORCE_PACK,
                              WIDE | binding.GALV_DP_NO_PACK, WIDE | binding.GALV_DP_NO_U32):
        check_against_oracle(w, flags=flags, table_instances=[0, 1, 2])


def test_degenerate_sizes():
    for (L, S, E) in [(1, 1, 0), (1, 7, 5), (6, 1, 15), (2, 3, 0), (3, 4, 1)]:
        w = workloads.random_workload(7, 4, L, S, E, m_range=(0, 3), c_range=(0, 5),
                                      r_range=(0, 5))
        w.budget[0] = E                     # at least one instance at the full width
        for flags in ALL_PATHS + (binding.GALV_DP_FORCE_PEEK, binding.GALV_DP_FORCE_PEEK | binding.GALV_DP_FORCE_PACK):
            check_against_oracle(w, flags=flags, table_instances=range(4))


def test_no_transition_selector_means_matrix_zero():
    w = workloads.random_workload(11, 2, 6, 5, 300, nR=2, m_range=(0, 60), c_range=(0, 99),
                                  r_range=(0, 99))
    sol = binding.Solver(w.B, w.L, w.S, w.E_max, w.nR)
    c, m, R, r_idx, budget = binding.upload(w)
    cost, _ = sol.solve(c, m, R, None, budget)
    plan = sol.backtrack()
    for b in range(w.B):
        ci, mi, Ri, _, bi = w.instance(b)
        ref = oracle.solve(ci, mi, Ri, None, bi)
        assert int(cost[b]) == ref.best_cost and (plan[b].cpu().numpy() == ref.plan).all()


def test_all_infeasible_and_huge_memory_values():
    w = workloads.random_workload(5, 3, 4, 6, 300, m_range=(30, 60), c_range=(1, 9), r_range=(0, 9))
    w.budget[:] = [300, 250, 119]                 # 119 < 4 * 30: nothing fits
    w.m[1, 2, :] = 2**31 - 1                      # a layer nobody can afford
    w.m[2, :, 0] = 2**31 - 1                      # strategy 0 never usable
    cost, last, plan, _ = check_against_oracle(w, table_instances=[0, 1, 2])
    assert cost[0] < INF
    for b in (1, 2):
        assert cost[b] == INF and last[b] == -1 and (plan[b] == -1).all()


def test_large_values_take_int64_path_and_agree():
    """Costs near 2^50 cannot be packed into a 52-bit key: the library must switch
    to the integer kernels by itself and still be exact."""
    w = workloads.random_workload(21, 4, 6, 10, 400, m_range=(0, 90), c_range=(0, 1 << 50),
                                  r_range=(0, 1 << 49))
    # instance 3 keeps small values: the choice is per instance
    w.c[3] = w.c[3] % 1000
    w.R[3] = w.R[3] % 1000
    cost, last, plan, status = check_against_oracle(w, table_instances=[0, 3])
    assert list(status) == [binding.GALV_INSTANCE_OK_INT64] * 3 + [binding.GALV_INSTANCE_OK_FAST_U32]


def test_mid_range_values_take_wide_storage():
    """Costs around 2^35 do not fit the 32-bit table cells but do fit a 52-bit key:
    the library keeps the packed-key kernels with 64-bit cells.  The last instance
    sits just below the narrow limit (sum of maxima + largest R < 2^31)."""
    w = workloads.random_workload(23, 4, 7, 12, 900, nR=2, m_range=(0, 150),
                                  c_range=(0, 1 << 35), r_range=(0, 1 << 33), infeasible=0.1)
    w.c[3] = w.c[3] % ((1 << 31) // 7 - (1 << 26))
    w.R[3] = w.R[3] % ((1 << 26) // 7)
    cost, last, plan, status = check_against_oracle(w, table_instances=[0, 1, 3])
    assert list(status) == [binding.GALV_INSTANCE_OK_FAST_WIDE] * 3 + [binding.GALV_INSTANCE_OK_FAST_U32]
    assert (cost[cost < INF] > (1 << 31)).any()


@pytest.mark.parametrize("S", [5, 22, 44, 100, 128, 200])
def test_large_costs_with_small_transition_costs_keep_32bit_keys(S):
    """Costs around 2^40 need 64-bit cells, but the keys hold only RELATIVE costs (clamped at the
    largest R + 1): with small transition costs the library keeps the 32-bit-key arithmetic and
    its pruning over 8-byte cells.  One instance keeps small costs (the choice is per instance);
    GALV_DP_NO_U32 sends the large ones to the 64-bit-key kernels instead."""
    w = workloads.random_workload(600 + S, 4, 6, S, 700, nR=2, m_range=(0, 150), c_range=(0, 1 << 40),
                                  r_range=(0, 3000), infeasible=0.08, zero_diagonal=False)
    w.c[3] = w.c[3] % 100000
    w.budget[:] = [700, 641, 577, 692]
    PACK, ROWS = binding.GALV_DP_FORCE_PACK, binding.GALV_DP_NO_PACK
    for peek in (binding.GALV_DP_FORCE_PEEK | PACK, binding.GALV_DP_NO_PEEK | PACK, binding.GALV_DP_FORCE_PEEK | ROWS,
                 binding.GALV_DP_NO_PEEK | ROWS, binding.GALV_DP_FORCE_PEEK | PACK | binding.GALV_DP_FORCE_WIDE_TILES):
        cost, _, _, status = check_against_oracle(w, flags=peek, table_instances=[0, 1, 3])
        assert list(status) == [binding.GALV_INSTANCE_OK_U32_WIDE] * 3 + [binding.GALV_INSTANCE_OK_FAST_U32]
        assert (cost[cost < INF] > (1 << 33)).any()
    _, _, _, status = check_against_oracle(w, flags=binding.GALV_DP_NO_U32, table_instances=[1])
    assert list(status) == [binding.GALV_INSTANCE_OK_FAST_WIDE] * 3 + [binding.GALV_INSTANCE_OK_FAST]
    check_against_oracle(w, flags=binding.GALV_DP_BP_U8 | binding.GALV_DP_STREAMS(2), table_instances=[2])


def test_wide_integer_keys_when_nothing_can_be_pruned_and_at_the_cost_limit():
    """Same path with transition costs above the cost spread (the kept-row list overflows: full
    loop over 8-byte cells) and with costs close to the 2^62 precondition."""
    w = workloads.random_workload(77, 3, 5, 44, 500, nR=2, m_range=(0, 120), c_range=(1 << 36, (1 << 36) + 9),
                                  r_range=(1000, 5000), infeasible=0.05, zero_diagonal=False)
    w.budget[0] = 500
    for flags in (binding.GALV_DP_FORCE_PEEK | binding.GALV_DP_FORCE_PACK, binding.GALV_DP_FORCE_PEEK | binding.GALV_DP_NO_PACK,
                  binding.GALV_DP_FORCE_PACK):
        _, _, _, status = check_against_oracle(w, flags=flags, table_instances=[0, 1, 2])
        assert (status == binding.GALV_INSTANCE_OK_U32_WIDE).all()
    w = workloads.random_workload(78, 2, 4, 9, 300, m_range=(0, 90), c_range=(0, (1 << 59) - 1), r_range=(0, 99))
    w.budget[0] = 300
    for flags in (binding.GALV_DP_FORCE_PACK, binding.GALV_DP_NO_PACK):
        cost, _, _, status = check_against_oracle(w, flags=flags, table_instances=[0, 1])
        assert (status == binding.GALV_INSTANCE_OK_U32_WIDE).all() and (cost[cost < INF] > (1 << 58)).any()


def test_path_limits_by_transition_cost():
    """32-bit integer keys need (2 * largest R + 2) * 2^k <= 2^32.  With k = 4: R up to 2^27 - 1 just
    fits; one more and the instance takes 64-bit keys (costs still fit 32-bit cells).  Clamping of
    relative costs is exercised hard here: R is far larger than the layer costs."""
    w = workloads.random_workload(31, 3, 4, 12, 700, nR=2, m_range=(0, 200), c_range=(0, 1000),
                                  r_range=(0, (1 << 27) - 1), infeasible=0.1, zero_diagonal=False)
    w.R[0, 1, 3, 5] = (1 << 27) - 1
    w.R[1, 0, 2, 2] = 1 << 27
    w.R[2] = w.R[2] % 50                         # tiny R: almost everything is clamped
    w.c[2] = w.c[2] * 1000
    cost, last, plan, status = check_against_oracle(w, table_instances=[0, 1, 2])
    assert list(status) == [binding.GALV_INSTANCE_OK_FAST_U32, binding.GALV_INSTANCE_OK_FAST,
                            binding.GALV_INSTANCE_OK_FAST_U32]


@pytest.mark.parametrize("L,expect", [(3, binding.GALV_INSTANCE_OK_FAST_U32), (6, binding.GALV_INSTANCE_OK_U32_WIDE)])
def test_largest_possible_key_is_a_candidate_but_never_a_stored_word(L, expect):
    """S = 16 (four index bits) and the largest R the 32-bit keys allow, 2^27 - 1: a former
    strategy 15 that is clamped (relative cost R_max + 1) and pays R_max yields the key 2^32 - 1,
    the very pattern the packed table uses for "unreachable".  It can never win (the strategy
    that attains the column's minimum offers a smaller key), so tables and plans must come out
    the same in both table forms."""
    rmax = (1 << 27) - 1
    w = workloads.random_workload(91, 2, L, 16, 500, nR=1, m_range=(0, 120), c_range=(0, 1000),
                                  r_range=(0, rmax), infeasible=0.05, zero_diagonal=False)
    w.R[:, 0, 15, :] = rmax                       # strategy 15 always pays the largest transition cost
    w.c[:, :, 15] += 2 * (1 << 27)                # ... and costs so much that it is clamped wherever another strategy fits
    w.budget[:] = [500, 377]
    for flags in (binding.GALV_DP_FORCE_PACK, binding.GALV_DP_NO_PACK, binding.GALV_DP_FORCE_PACK | binding.GALV_DP_FORCE_PEEK):
        check_against_oracle(w, flags=flags, table_instances=[0, 1], expect_status=expect)


def test_bad_values_are_reported_not_solved():
    w = workloads.random_workload(3, 5, 4, 5, 50, m_range=(0, 9), c_range=(0, 9), r_range=(0, 9))
    w.c[0, 1, 2] = -1
    w.m[1, 0, 0] = -5
    w.R[2, 0, 1, 3] = 1 << 62
    w.budget[3] = 51
    cost, last, plan, status, _ = gpu_solve(w)
    assert list(status[:4]) == [binding.GALV_INSTANCE_BAD_VALUE] * 4
    assert (cost[:4] == INF).all() and (last[:4] == -1).all() and (plan[:4] == -1).all()
    ref = oracle.solve(*w.instance(4))
    assert status[4] == binding.GALV_INSTANCE_OK_FAST_U32 and cost[4] == ref.best_cost


def test_call_order_and_reuse():
    w = workloads.random_workload(9, 2, 5, 6, 200, m_range=(0, 40), c_range=(0, 99), r_range=(0, 99))
    sol = binding.Solver(w.B, w.L, w.S, w.E_max, w.nR)
    with pytest.raises(binding.GalvError) as ei:
        sol.backtrack()
    assert ei.value.code == binding.GALV_ERR_STATE
    dev = binding.upload(w)
    first = [t.clone() for t in sol.solve(*dev)] + [sol.backtrack().clone()]
    # a different problem through the same handle, then the first one again
    w2 = workloads.random_workload(10, 2, 5, 6, 200, m_range=(0, 40), c_range=(0, 99), r_range=(0, 99))
    sol.solve(*binding.upload(w2))
    again = list(sol.solve(*dev)) + [sol.backtrack()]
    for x, y in zip(first, again):
        assert torch.equal(x, y)
    with pytest.raises(binding.GalvError):
        sol.export_tables(5)


def test_one_handle_through_every_storage_form():
    """The same handle solves, in turn, problems that land on different arithmetic paths and
    table forms (single packed table, narrow and wide cost rows with their infinity leads,
    64-bit integers): whatever one solve leaves in the workspace must not leak into the next."""
    shape = dict(B=3, L=6, S=23, E_max=900, nR=2)
    kinds = {
        "packed": dict(c_range=(0, 5000), r_range=(0, 300)),
        "narrow rows": dict(c_range=(0, 5000), r_range=(0, 1 << 28)),
        "packed, 64-bit minima": dict(c_range=(0, 1 << 40), r_range=(0, 300)),
        "wide rows": dict(c_range=(0, 1 << 36), r_range=(0, 1 << 34)),
        "int64": dict(c_range=(0, 1 << 58), r_range=(0, 1 << 57)),
    }
    expect = {"packed": binding.GALV_INSTANCE_OK_FAST_U32, "narrow rows": binding.GALV_INSTANCE_OK_FAST,
              "packed, 64-bit minima": binding.GALV_INSTANCE_OK_U32_WIDE, "wide rows": binding.GALV_INSTANCE_OK_FAST_WIDE,
              "int64": binding.GALV_INSTANCE_OK_INT64}
    order = ["packed", "narrow rows", "packed", "packed, 64-bit minima", "wide rows", "packed, 64-bit minima",
             "narrow rows", "int64", "packed", "wide rows", "packed"]
    for flags in (binding.GALV_DP_FORCE_PEEK | binding.GALV_DP_FORCE_PACK, binding.GALV_DP_FORCE_PACK,
                  binding.GALV_DP_NO_PACK):
        sol = binding.Solver(shape["B"], shape["L"], shape["S"], shape["E_max"], shape["nR"], flags)
        for step, kind in enumerate(order):
            w = workloads.random_workload(7000 + step, shape["B"], shape["L"], shape["S"], shape["E_max"], nR=2,
                                          m_range=(0, 200), infeasible=0.08, zero_diagonal=False, **kinds[kind])
            w.budget[0] = shape["E_max"]
            cost, last = sol.solve(*binding.upload(w))
            plan = sol.backtrack()
            assert (sol.status().cpu().numpy() == expect[kind]).all(), (step, kind)
            for b in range(w.B):
                ref = oracle.solve(*w.instance(b), want_C_last=True, want_bp=True)
                assert int(cost[b]) == ref.best_cost and int(last[b]) == ref.best_last, (step, kind, b)
                assert (plan[b].cpu().numpy() == ref.plan).all(), (step, kind, b)
                C, bp = sol.export_tables(b)
                Eb = int(w.budget[b])
                assert (C.cpu().numpy()[:Eb + 1] == ref.C_last).all(), (step, kind, b)
                assert (bp.cpu().numpy()[:, :Eb + 1] == ref.bp).all(), (step, kind, b)
        sol.close()


def test_runs_on_a_side_stream():
    w = workloads.config(1, 2)
    sol = binding.Solver(w.B, w.L, w.S, w.E_max, w.nR)
    dev = binding.upload(w)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        cost, _ = sol.solve(*dev)
        plan = sol.backtrack()
    side.synchronize()
    for b, ref in enumerate(oracle.solve_workload(w, threads=2)):
        assert int(cost[b]) == ref.best_cost and (plan[b].cpu().numpy() == ref.plan).all()


# ------------------------------------------------------------------ size limits

@pytest.mark.parametrize("S", [513, 1024])
def test_maximum_strategy_counts(S):
    """Up to the documented limit of 1024 strategies (32 strategy-group blocks along grid.y,
    10 index bits in the key), both arithmetic paths, exported tables included."""
    w = workloads.random_workload(S, 2, 3, S, 300, nR=2, m_range=(0, 120), c_range=(0, 30),
                                  r_range=(0, 12), infeasible=0.05, zero_diagonal=False)
    w.budget[0] = 300
    for flags in ALL_PATHS:
        check_against_oracle(w, flags=flags, table_instances=[0])


def test_very_wide_budget_axis():
    """2^20 budget columns (8192 budget tiles), two strategies: every column against the oracle."""
    E = 1 << 20
    w = workloads.random_workload(3, 2, 4, 2, E, m_range=(0, E // 3), c_range=(0, 1000), r_range=(0, 50),
                                  budgets=[E, E - 12345])
    check_against_oracle(w, table_instances=[0, 1])
    check_against_oracle(w, flags=binding.GALV_DP_BP_U8 | binding.GALV_DP_STREAMS(2), table_instances=[1])


def test_many_tiny_instances():
    """4000 instances in one launch (grid.z), ragged budgets, internal streams by the shape's default and forced."""
    w = workloads.random_workload(12, 4000, 5, 6, 90, m_range=(0, 30), c_range=(0, 40), r_range=(0, 9),
                                  infeasible=0.1)
    for flags in (0, binding.GALV_DP_STREAMS(7)):
        cost, last, plan, _ = check_against_oracle(w, flags=flags, threads=8)
        check_properties(w, cost, last, plan)
