#!/usr/bin/env python3
"""Benchmark of the batched plan-search dynamic program on one MI355X.

One "step" is one pass of the whole hot path over one batch of synthetic search
instances that already live in HBM: galv_dp_solve_batched (preparation, layer 0,
the L-1 layer sweeps, final minimum) followed by galv_dp_backtrack.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config N] [--no-cpu-baseline]
                    [--streams N] [--bp-u8] [--graph] [--no-extra-legs] [--coarsen FUSE,GRAN]

Prints ONE JSON line.  By default both target configurations are timed, 4 (the
largest that one GPU holds: the headline `value`, `ms_per_step`, `roofline` and
`cpu_baseline`) and 3; `per_config` carries the full record of each.  `--config N`
times that configuration alone.  `value` is DP cell-updates/s with the metric's
nominal count sum_b L * E_b * S^2 per batch, in the library's default
configuration (int32 back-pointers, internal streams chosen from the shape);
searches/s and the exact candidate rate are reported beside it.

`roofline` is for the layer-sweep kernel (the only kernel that matters: > 95 %
of the time).  Two sides are computed per layer step, and the one that needs
more time at its peak is the binding one (`roofline.bound`):
  * HBM: the table bytes of a state within the budgets, against 8 TB/s.  With the
    single packed table (the library's choice when a layer fills the chip, as on
    configurations 2-4) that is 8 bytes: one 32-bit word read and one written,
    the word holding the back-pointer and the cost relative to its column's
    former minimum, plus one minimum per budget column.  With rolling cost rows
    (small shapes, --no-pack, one-byte back-pointers) it is 12: cost cell read,
    cost cell written, int32 back-pointer written (20 with 64-bit cells);
  * ALU: the min-plus candidates the sweep evaluates (the library counts them:
    on the 32-bit-key path former strategies that cannot win any minimum of a
    tile are pruned; `candidates_evaluated_share`) times the lane-operations
    each needs on its instance's arithmetic path (1.5 with 32-bit keys: two adds
    and one three-way minimum per two candidates; 2 with 64-bit keys), plus 7 per
    table state on the 32-bit-key path, against the VALU issue peak of
    256 CUs x 64 lanes x 2.4 GHz = 39.3 T lane-ops/s.
The sweep time per layer comes from events on the caller's stream around the
solve, / (L-1).  With internal streams a layer is several overlapping launches,
so that figure rests on event timing; `roofline.single_stream` is a second timed
leg with one launch per layer, the kernel's own figure, which a kernel trace of
`--streams 1` shows directly.
`variant_bp_u8` is a third leg with one-byte back-pointers (same results; rolling
cost rows, 9 B/state: it saves workspace, not time, where the packed table applies).
`cpu_baseline` times the serial CPU oracle (test infrastructure, never tuned) on a
bounded sample of the same workload: one instance on one thread, and one instance
per thread on the host cores this process may use.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

VALU_PEAK_TLANEOPS = 256 * 64 * 2.4e9 / 1e12      # 39.3
HBM_PEAK_GBS = 8000.0
# VALU lane-operations one min-plus candidate needs, by the arithmetic path of its instance
# (status code): 32-bit keys fold two candidates into two adds and one three-way minimum;
# 64-bit keys take one add and one minimum each; the general integer path about six.
OPS_PER_CANDIDATE = {3: 1.5, 4: 1.5, 0: 2.0, 2: 2.0, 1: 6.0}
# lane-operations per table state that do not depend on the number of candidates, 32-bit-key path:
# column minimum (1), relative cost and clamp test (2), new cell and back-pointer (4)
FIXED_OPS_PER_STATE = {3: 7.0, 4: 12.0}
# table bytes per state: cost cell read + cost cell written + int32 back-pointer written
BYTES_PER_STATE = {3: 4 + 4 + 4, 0: 4 + 4 + 4, 4: 8 + 8 + 4, 2: 8 + 8 + 4, 1: 8 + 8 + 4}   # by per-instance status code


# HBM bytes per sweep launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, each scaled by the
# same counter's reading for a 1 GiB copy: the `traffic_bytes_per_launch` line of
# profiles/sweep_kernel_config<N>.md (tests/test_profiles.py keeps the two equal); None where not measured.
MEASURED_TRAFFIC_BYTES = {3: 322060786, 4: 659360817}


def cpu_baseline(w):
    """Oracle wall time on a bounded sample of the workload's instances: one instance on one
    thread (per-core rate), then one instance per thread side by side (whole-host rate).
    An instance whose full budget would take the oracle minutes is solved at a truncated
    budget (same layers, strategies and values; the work per budget column does not depend on
    the column), and the sample says so."""
    import copy

    import oracle
    oracle.build()
    host = os.cpu_count() or 1
    try:
        host = min(host, len(os.sched_getaffinity(0)))
    except (AttributeError, OSError):
        pass
    # a GPU machine gives one GPU's job a share of 16 cores whatever the core count it shows
    threads = max(1, min(host, 16, w.B))
    per_core = 2.0e9                                   # rough oracle rate used only to size the sample
    cap = int(15.0 * per_core / (w.L * w.S * w.S))     # budget columns one thread sweeps in ~15 s
    ws = copy.copy(w)
    ws.budget = w.budget.copy()
    truncated = bool((ws.budget > cap).any())
    ws.budget[ws.budget > cap] = cap
    ids = sorted({int(round(i * (w.B - 1) / max(1, threads - 1))) for i in range(threads)})
    updates = lambda b: w.L * int(ws.budget[b]) * w.S * w.S
    what = (f"budgets truncated to {cap} of {int(w.budget.max())} columns" if truncated
            else "full budget each")
    one = ids[len(ids) // 2]
    t0 = time.perf_counter()
    oracle.solve_workload(ws, [one], threads=1)
    dt1 = time.perf_counter() - t0
    t0 = time.perf_counter()
    oracle.solve_workload(ws, ids, threads=len(ids))
    dt = time.perf_counter() - t0
    return {"value": sum(updates(b) for b in ids) / dt, "unit": "cell-updates/s", "cores": len(ids),
            "host_cpu_count": os.cpu_count(), "kind": "oracle", "seconds": round(dt, 3),
            "sample": f"{len(ids)} of {w.B} instances of '{w.name}' (ids {ids}), one per thread, "
                      f"all L layers, {what}",
            "single_thread": {"value": updates(one) / dt1, "unit": "cell-updates/s", "cores": 1,
                              "seconds": round(dt1, 3),
                              "sample": f"instance {one} of '{w.name}', all L layers, {what}"}}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--config", type=int, default=None,
                    help="workload index 0..4; default: 4 (headline) and 3, both target configurations")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--force-int64", action="store_true", help="time the general integer kernels")
    ap.add_argument("--no-u32", action="store_true", help="keep 64-bit keys (GALV_DP_NO_U32)")
    ap.add_argument("--no-pack", action="store_true",
                    help="rolling cost rows and plain back-pointers instead of the single packed table (GALV_DP_NO_PACK)")
    ap.add_argument("--force-pack", action="store_true", help="the single packed table whatever the shape (GALV_DP_FORCE_PACK)")
    ap.add_argument("--no-wide-tiles", action="store_true", help="128-column tiles whatever the shape (GALV_DP_NO_WIDE_TILES)")
    ap.add_argument("--bp-u8", action="store_true",
                    help="store back-pointers in one byte (GALV_DP_BP_U8): 9 instead of 12 B per state")
    ap.add_argument("--streams", type=int, default=0,
                    help="internal streams the layer sweeps are spread over (0 = library's choice, 1 = none)")
    ap.add_argument("--no-extra-legs", action="store_true",
                    help="time only the main configuration (skip the single-stream and one-byte legs), "
                         "so that a profile of the run holds one kind of launch")
    ap.add_argument("--coarsen", default=None, metavar="FUSE,GRAN",
                    help="instead of the main benchmark: time the coarse-grained search (layers fused in groups "
                         "of FUSE, memory in units GRAN times larger) and report its cost error against the "
                         "fine-grained optimum of the same instances")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step (solve + backtrack) into a HIP graph and time replays of it: "
                         "removes the host's per-launch cost, which dominates the small configurations")
    ap.add_argument("--alg1", default=None, metavar="LAYERS,DEVICES,BUDGET",
                    help="instead of the main benchmark: time Algorithm 1 (windowed driver over the batched "
                         "solver) on a seeded synthetic cost model and the plain oracle loop beside it")
    ap.add_argument("--c-scale", type=int, default=1,
                    help="multiply every layer cost AND transition cost by this factor (not the named configuration "
                         "any more): large costs need 64-bit table cells")
    ap.add_argument("--r-scale", type=int, default=1,
                    help="multiply every transition cost by this factor (not the named configuration any more): "
                         "with transition costs far above the spread of the layer costs nothing can be pruned, "
                         "which is the sweep's worst case")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a kernel of known traffic: 1 GiB read, "
                         "1 GiB written) so that rocprofv3 FETCH_SIZE / WRITE_SIZE readings can be scaled")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU; instances are independent, so more GPUs "
              "would just split the batch (no multi-GPU path is part of it). Use --gpus 1.",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2211_13878_amd import binding, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    if args.alg1:
        from paper_2211_13878_amd import alg1
        n_layers, n_dev, budget = (int(x) for x in args.alg1.split(","))
        model = workloads.Alg1Model(42, n_layers, n_dev, alg1.strategy_counts(n_dev))
        sizes = range(1, 100000)
        for _ in range(max(1, args.warmup)):
            res = alg1.optimize(model, n_dev, budget, sizes)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            res = alg1.optimize(model, n_dev, budget, sizes)
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        n_dp = (res.n_explored + 1) * (2 * n_dev - 1)          # one search per batch size, degree and stage
        out = {"metric": "alg1_optimizations", "ms_per_step": ms,
               "config": {"workload": f"Algorithm 1, synthetic cost model seed 42, L={n_layers}, N={n_dev}, "
                                      f"budget {budget} units, batch sizes 1, 2, ... until Out-Of-Memory"},
               "batch_sizes_explored": res.n_explored, "searches_needed": n_dp,
               "searches_per_sec": n_dp / (ms * 1e-3), "best": [res.batch, res.pp, res.cost]}
        if not args.no_cpu_baseline:
            import oracle
            from oracle import alg1 as oracle_alg1
            oracle.build()
            t0 = time.perf_counter()
            ref = oracle_alg1.optimize(model, n_dev, budget, sizes)
            dt = time.perf_counter() - t0
            assert (ref["batch"], ref["pp"], ref["cost"]) == (res.batch, res.pp, res.cost)
            out["cpu_baseline"] = {"ms": dt * 1e3, "cores": 1, "kind": "oracle"}
        print(json.dumps(out))
        return

    configs = [args.config] if args.config is not None else [4, 3]
    if args.coarsen:
        cfg = configs[-1]
        w = workloads.config(cfg)
        dev = binding.upload(w)
        torch.cuda.synchronize()
        fuse, gran = (int(x) for x in args.coarsen.split(","))
        fine = binding.Solver(w.B, w.L, w.S, w.E_max, w.nR)
        fine.solve(*dev)
        fine_cost = fine.best_cost.cpu().numpy()
        fine.close()
        del fine
        torch.cuda.empty_cache()
        Lc = (w.L + fuse - 1) // fuse
        sol = binding.Solver(w.B, Lc, w.S, w.E_max // gran, w.nR)

        def coarse_step():
            c2, m2, r2, e2 = binding.galv_dp_coarsen(fuse, gran, *dev)
            sol.solve(c2, m2, dev[2], r2, e2)
            return binding.galv_dp_expand_plan(sol.backtrack(), w.L, fuse)

        for _ in range(args.warmup):
            coarse_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            coarse_step()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) * 1e3 / args.steps
        cost = sol.best_cost.cpu().numpy()
        both = (fine_cost < binding.GALV_INF) & (cost < binding.GALV_INF)
        rel = (cost[both] - fine_cost[both]) / fine_cost[both]
        print(json.dumps({
            "metric": "coarsened_search", "config": {"workload": f"config {cfg} '{w.name}'",
                                                      "fuse": fuse, "granularity": gran},
            "ms_per_step": ms, "searches_per_sec": w.B / (ms * 1e-3),
            "layers": [w.L, Lc], "budget_columns": [w.E_max + 1, w.E_max // gran + 1],
            "feasible_fine": int((fine_cost < binding.GALV_INF).sum()),
            "feasible_coarse": int((cost < binding.GALV_INF).sum()),
            "cost_error_mean": float(rel.mean()) if rel.size else None,
            "cost_error_max": float(rel.max()) if rel.size else None}))
        return


    records = {cfg: run_config(cfg, args, torch, binding, workloads) for cfg in configs}
    out = dict(records[configs[0]])           # the headline: the first configuration timed
    if len(configs) > 1:
        out["per_config"] = {str(cfg): rec for cfg, rec in records.items()}
    print(json.dumps(out))


def run_config(cfg, args, torch, binding, workloads):
    """Time one named configuration; returns its record (the JSON line's fields)."""
    w = workloads.config(cfg)
    if args.r_scale != 1:
        w.R = w.R * args.r_scale
        w.name += f" with R x {args.r_scale}"
    if args.c_scale != 1:
        w.R = w.R * args.c_scale
        w.c = w.c * args.c_scale
        w.name += f" with c and R x {args.c_scale}"
    base_flags = ((binding.GALV_DP_FORCE_INT64 if args.force_int64 else 0) |
                  (binding.GALV_DP_NO_U32 if args.no_u32 else 0) |
                  (binding.GALV_DP_NO_PACK if args.no_pack else 0) |
                  (binding.GALV_DP_FORCE_PACK if args.force_pack else 0) |
                  (binding.GALV_DP_NO_WIDE_TILES if args.no_wide_tiles else 0) |
                  (binding.GALV_DP_BP_U8 if args.bp_u8 else 0))
    dev = binding.upload(w)
    torch.cuda.synchronize()

    if args.calibrate_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    chosen = {}       # what the handle of the last timed leg chose (packed table, peek, streams)

    def timed(flags, steps, warmup):
        """K steps (solve + backtrack) on a fresh handle: wall ms per step, solve ms per step."""
        sol = binding.Solver(w.B, w.L, w.S, w.E_max, w.nR, flags)
        for _ in range(warmup):
            sol.solve(*dev)
            sol.backtrack()
        torch.cuda.synchronize()
        # Events sit on torch's current stream, which is the stream the binding hands to the
        # library; the library joins its internal streams back into it before the final
        # minimum, so the events bracket all of a solve's launches.
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
              for _ in range(steps)]
        graph = None
        if args.graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph):
                sol.solve(*dev)
                sol.backtrack()
            graph.replay()
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for a, b in ev:
            a.record()
            if graph is not None:
                graph.replay()          # the events then bracket solve + backtrack (< 1 % more)
                b.record()
                continue
            sol.solve(*dev)
            b.record()
            sol.backtrack()
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
        solve_ms = sorted(a.elapsed_time(b) for a, b in ev)
        status = sol.status().cpu().numpy()
        stats = sol.stats().cpu().numpy()
        cost = sol.best_cost.cpu().numpy()
        chosen.update(sol.config())
        sol.close()
        del sol
        torch.cuda.empty_cache()
        return wall * 1e3 / steps, solve_ms, status, cost, stats

    nominal = w.nominal_cell_updates()
    exact = w.exact_candidates()
    states = w.n_states()
    n_layer_steps = max(1, w.L - 1)

    def alu(solve_ms):
        """Sweep lane-ops per layer step over its duration (prep / init / final are < 1 % and
        counted into the duration, so this is a lower bound)."""
        layer_ms = sum(solve_ms) / len(solve_ms) / n_layer_steps
        achieved = lane_ops_per_layer / (layer_ms * 1e-3) / 1e12
        return layer_ms, achieved

    ms_per_step, solve_ms, status, cost, stats = timed(base_flags | binding.GALV_DP_STREAMS(args.streams),
                                                       args.steps, args.warmup)
    main_leg = dict(chosen)
    # Share of the min-plus candidates the sweep evaluated: on the 32-bit-key path rows that cannot
    # win any minimum of a tile are left out (the library counts rows reduced / rows listed).
    share = [float(r) / float(n) if n > 0 else 1.0 for r, n, _ in stats]
    fetched_share = (float(sum(f for _, _, f in stats)) / float(sum(n for _, n, _ in stats))
                     if sum(n for _, n, _ in stats) > 0 else 1.0)
    # lane-ops of one layer: per instance and table state the fixed work of its path, plus its
    # (E_b + 1) * S^2 candidates, as far as they were evaluated, times the path's cost per candidate
    lane_ops_per_layer = sum((FIXED_OPS_PER_STATE.get(int(st), 0.0) +
                              f * w.S * OPS_PER_CANDIDATE.get(int(st), 0.0)) * (int(e) + 1) * w.S
                             for st, e, f in zip(status, w.budget, share))
    evaluated = sum(f * (int(e) + 1) * w.S * w.S for e, f in zip(w.budget, share))     # per layer
    ops = OPS_PER_CANDIDATE.get(int(status[0]), 0.0)
    sweep_ms, achieved = alu(solve_ms)
    # single packed table (the library's default with int32 back-pointers and S <= 256): 32-bit-key instances
    # read and write one 4-byte word per state, plus one former minimum per budget column
    packed = bool(main_leg["packed"])
    per_state = [(4 + 4 + 2 * (4 if int(st) == 3 else 8) / w.S) if packed and int(st) in (3, 4)
                 else BYTES_PER_STATE.get(int(st), 0) - (3 if args.bp_u8 else 0) for st in status]
    hbm_bytes = sum(p * (int(e) + 1) * w.S for p, e in zip(per_state, w.budget))   # per layer
    hbm_gbs = hbm_bytes / (sweep_ms * 1e-3) / 1e9
    # The same kernel with every layer as ONE launch on one stream: the per-launch figure that
    # a kernel trace shows directly (with several streams the launches overlap in time).
    single = None
    if not args.no_extra_legs:
        _, solve_ms_1, _, _, _ = timed(base_flags | binding.GALV_DP_STREAMS(1), max(2, args.steps // 2), 1)
        launch_ms_1, achieved_1 = alu(solve_ms_1)
        single = {"launch_ms": launch_ms_1,
                  "alu": {"achieved": achieved_1, "frac": achieved_1 / VALU_PEAK_TLANEOPS},
                  "hbm": {"achieved": hbm_bytes / (launch_ms_1 * 1e-3) / 1e9,
                          "frac": hbm_bytes / (launch_ms_1 * 1e-3) / 1e9 / HBM_PEAK_GBS}}

    # Which roofline binds: the one that needs more time at its peak for one layer's work.
    alu_obj = {"achieved": achieved, "peak": VALU_PEAK_TLANEOPS, "unit": "Tlane-op/s",
               "frac": achieved / VALU_PEAK_TLANEOPS, "lane_ops_per_candidate": ops,
               "lane_ops_per_state_fixed": FIXED_OPS_PER_STATE.get(int(status[0]), 0.0),
               "candidates_evaluated_share": evaluated / max(1.0, exact / n_layer_steps)}
    hbm_obj = {"achieved": hbm_gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": hbm_gbs / HBM_PEAK_GBS,
               "bytes_per_launch": hbm_bytes, "bytes_per_state": max(per_state)}
    t_alu = lane_ops_per_layer / (VALU_PEAK_TLANEOPS * 1e12)
    t_hbm = hbm_bytes / (HBM_PEAK_GBS * 1e9)
    bound = "alu" if t_alu >= t_hbm else "hbm"
    binding_obj = alu_obj if bound == "alu" else hbm_obj
    roofline = {"bound": bound, "kernel": "sweep_kernel", "achieved": binding_obj["achieved"],
                "peak": binding_obj["peak"], "unit": binding_obj["unit"], "frac": binding_obj["frac"],
                "traffic": (MEASURED_TRAFFIC_BYTES.get(cfg) if base_flags == 0 and args.r_scale == 1 and args.c_scale == 1
                            else None),
                "launch_ms": sweep_ms,
                "time_at_peak_us": {"alu": t_alu * 1e6, "hbm": t_hbm * 1e6},
                "note": "per layer step of the whole batch, from events on the caller's stream around the "
                        "solve; with internal streams a layer step is several overlapping launches, so this "
                        "figure rests on event timing only; single_stream is the kernel's own figure (one "
                        "launch per layer, the duration a kernel trace of --streams 1 shows). The ALU side "
                        "counts only the candidates the sweep evaluates (rows that cannot win any minimum "
                        "of a tile are pruned; alu.candidates_evaluated_share, from galv_dp_get_stats)",
                "single_stream": single, "alu": alu_obj, "hbm": hbm_obj}

    kinds = {3: "u32", 4: "u32", 0: "f64", 2: "f64", 1: "int64"}
    used = sorted({kinds[int(st)] for st in status if int(st) in kinds})
    dtype = ("+".join(used) or "none") + " (exact integer keys; int64 costs in, int64 costs out)"

    out = {
        "metric": "dp_cell_updates_per_sec",
        "value": nominal / (ms_per_step * 1e-3),
        "unit": "cell-updates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": dtype,
        "data": "synthetic",
        "config": {"workload": f"config {cfg} '{w.name}': B={w.B} L={w.L} S={w.S} "
                               f"E_max={w.E_max} budgets {int(w.budget.min())}..{int(w.budget.max())}",
                   "back_pointer_bytes": 1 if args.bp_u8 else 4,
                   "single_packed_table": bool(packed and any(int(st) in (3, 4) for st in status)),
                   "internal_streams": main_leg["streams"],
                   "peek_before_fetch": bool(main_leg["peek"]),
                   "tile_columns": main_leg["tile_columns"],
                   "hip_graph_replay": bool(args.graph),
                   "cell_updates_per_batch": nominal, "exact_candidates_per_batch": exact,
                   "table_states_per_batch": states},
        "searches_per_sec": w.B / (ms_per_step * 1e-3),
        "exact_candidates_per_sec": exact / (ms_per_step * 1e-3),
        "candidates_evaluated_share": evaluated / max(1.0, exact / n_layer_steps),
        "cost_rows_fetched_share": fetched_share,
        "solve_ms_median": solve_ms[len(solve_ms) // 2],
        "instances_by_path": {"u32_keys": int((status == binding.GALV_INSTANCE_OK_FAST_U32).sum()),
                              "u32_keys_64bit_cells": int((status == binding.GALV_INSTANCE_OK_U32_WIDE).sum()),
                              "f64_keys_32bit_cells": int((status == binding.GALV_INSTANCE_OK_FAST).sum()),
                              "f64_keys_64bit_cells": int((status == binding.GALV_INSTANCE_OK_FAST_WIDE).sum()),
                              "int64": int((status == binding.GALV_INSTANCE_OK_INT64).sum())},
        "instances_feasible": int((cost < binding.GALV_INF).sum()),
        "roofline": roofline,
    }
    if not (args.bp_u8 or args.force_int64 or args.no_extra_legs) and w.S <= 255:
        # storage variant, same results: one-byte back-pointers (rolling cost rows, 9 B per state)
        ms_u8, _, _, cost_u8, _ = timed(binding.GALV_DP_BP_U8 | binding.GALV_DP_STREAMS(args.streams),
                                     max(2, args.steps // 2), 1)
        assert (cost_u8 == cost).all()
        out["variant_bp_u8"] = {"ms_per_step": ms_u8, "value": nominal / (ms_u8 * 1e-3)}
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    del dev
    torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
