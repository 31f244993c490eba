#!/usr/bin/env python3
"""Benchmark of the allocation search on one MI355X.

A step is one pass of the whole hot path (cost table, prune, plan, enumeration
with fused arg-min, finalize) over one synthetic workload whose tables are
already resident in HBM.  Default workload: the 8-task XR-shaped graph with a
64-level demand sweep, pruned to <= 20 choices per task (up to 20^8 candidates
per level), seed 0.

Prints one JSON line: candidates evaluated per second, the enumeration kernel's
fraction of the VALU roofline, and the CPU oracle timed on a bounded sample.
The headline numbers are those of the plain enumeration, in which the tests of
every candidate are issued; the library's default search, which leaves out what
latency and capacity bounds exclude in bulk and returns the same results, is timed
right after it and reported under "with_bounds".
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Algorithmic vector lane-operations of the enumeration, counted for the sharing the
# kernel does: per candidate one latency compare and one minimum on its key.  The
# accuracy test is shared by all candidates of one pair of variants of the two innermost
# tasks (and one combination of the others) and is left out, like everything shared further
# out, so the figure is a lower bound of what the kernel issues.
OPS_PER_CANDIDATE = 2
# The rule of the previous kernel, which tested the accuracy once per (variant of the innermost
# task, combination of all other tasks): two more lane-operations per such group.  Reported
# beside the headline fraction so that the two kernels can be compared under one rule (the
# present kernel no longer issues those operations, so the figure can pass 1).
OPS_PER_VARIANT_GROUP = 2
# For comparison, a count that charges every candidate its own arithmetic: cost add,
# latency add, fma, three compares, two mask ANDs, three for the running minimum.
UNSHARED_OPS_PER_CANDIDATE = 11
# HBM bytes per launch of the enumeration kernel, from rocprofv3 FETCH_SIZE / WRITE_SIZE scaled
# against a 1 GiB copy (profiles/enumerate_kernel_xr8_hbm_traffic.md); known only for the
# default workload in cost mode.
# key: workload, seed, objective mode, mixture mode, bounds
MEASURED_TRAFFIC_BYTES = {("xr8", 0, False, False, False): (18059 + 8614) * 1024,
                          ("xr8", 0, False, False, True): (6631 + 1603) * 1024}
# SQ counters of the same launch (profiles/enumerate_kernel_xr8_counters.md): vector instructions
# issued per candidate (wave instructions x 64 lanes / candidates) and VALU issue utilisation
# (wave instructions x 4 cycles / (SIMDs x elapsed cycles)); same key as above
MEASURED_COUNTERS = {("xr8", 0, False, False, False): {"valu_lane_ops_per_candidate": 2.20, "issue_utilisation": 0.99,
                                                       "scalar_instructions_per_cu_cycle": 0.38,
                                                       "source": "profiles/enumerate_kernel_xr8_counters.md"},
                     ("xr8", 0, False, False, True): {"valu_lane_ops_per_scored_candidate": 35.9, "issue_utilisation": 0.71,
                                                      "source": "profiles/enumerate_kernel_xr8_counters.md"},
                     ("xr8", 0, True, False, False): {"valu_lane_ops_per_candidate": 2.74, "issue_utilisation": 0.98,
                                                      "source": "profiles/enumerate_kernel_xr8_counters.md"}}
# 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz: one full-rate VALU lane-op per lane per cycle
VALU_PEAK_LANE_OPS = 256 * 4 * 16 * 2.4e9


def peak_probe():
    """Sustained lane-operations/s of dependent-free instruction streams on this GPU
    (paper_2603_08797_amd/csrc/peak_probe.hip, a library of its own): what the vector ALUs deliver
    at the clock they hold under load, beside the 2.4 GHz paper figure.  v_min_u32 and
    v_cmp_le_u32 are the two instructions the enumeration spends per candidate; v_add_u32 issues
    at a higher rate that those two do not reach."""
    import ctypes as C
    path = os.path.join(ROOT, "paper_2603_08797_amd", "libjsv_probe.so")
    if not os.path.exists(path):
        return None
    lib = C.CDLL(path)
    lib.jsv_probe_valu.restype = C.c_int
    lib.jsv_probe_valu.argtypes = [C.c_int, C.c_uint32, C.c_uint32, C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    out = {"unit": "Tlane-op/s", "paper_peak": VALU_PEAK_LANE_OPS / 1e12}
    for kind, name in ((0, "v_add_u32"), (2, "v_min_u32"), (3, "v_cmp_le_u32"), (1, "v_fma_f64")):
        sec, ops = C.c_double(), C.c_double()
        rc = lib.jsv_probe_valu(kind, 256 * 8, 6000, 5, C.byref(sec), C.byref(ops))
        if rc != 0 or sec.value <= 0:
            out[name] = None
            continue
        out[name] = ops.value / sec.value / 1e12
        out[name + "_ms"] = sec.value * 1e3
    return out


# Mixture mode: every option has its own accuracy, so each candidate is charged its latency
# compare, its fma, its accuracy compare and its minimum.
OPS_PER_CANDIDATE_MIXTURES = 4


def algorithmic_ops(results, mixtures=False):
    """Lane-ops per step by the rule above."""
    return float(sum(r.evaluated for r in results) * (OPS_PER_CANDIDATE_MIXTURES if mixtures else OPS_PER_CANDIDATE))


def previous_rule_ops(jsv_mod, problems, searches, results, factors=None, mixtures=False):
    """Lane-ops per step by the previous kernel's rule; needs K and the number of surviving
    variants of the innermost task (the lowest-numbered source) at every level."""
    total = 0.0
    if mixtures:
        return float(sum(r.evaluated for r in results) * OPS_PER_CANDIDATE_MIXTURES)
    if factors is not None:
        # exhaustive search with per-variant factors: the innermost task is held to one variant
        # per combination if its outgoing factors differ between variants, else it keeps all V
        pb, se = problems[0], searches[0]
        if se.prune_cap != 0:
            return None
        has_pred = set(int(x) for x in pb.dst.tolist())
        t0 = min(t for t in range(pb.T) if t not in has_pred)
        held = any(int(a) == t0 and len(set(factors[e].tolist())) > 1 for e, a in enumerate(pb.src.tolist()))
        groups, K = (1, pb.P * pb.B) if held else (pb.V, pb.C)
        return sum(r.evaluated for r in results) * (OPS_PER_CANDIDATE + OPS_PER_VARIANT_GROUP * groups / K)
    ctx = jsv_mod.Jsv(device=0)
    k = 0
    for pb, se in zip(problems, searches):
        has_pred = set(int(x) for x in pb.dst.tolist())
        t0 = min(t for t in range(pb.T) if t not in has_pred)
        ctx.load(pb)
        for D in se.demand_mrps.tolist():
            n = results[k].evaluated
            k += 1
            if n == 0:
                continue
            ids, _ = ctx.get_pruned(D, se.slo_latency_us, se.prune_cap, t0)
            groups = len(set(int(c) // (pb.P * pb.B) for c in ids.tolist()))
            total += n * (OPS_PER_CANDIDATE + OPS_PER_VARIANT_GROUP * groups / len(ids))
    ctx.close()
    return total


PAPER_CONTEXT = ("paper (other hardware, context only): MILP solve 2-20 s per invocation on a 96-core "
                 "host (Gurobi); 11.3x max serviceable demand vs closest prior work (analytical, 840 "
                 "H100 MIG slices); 43.3% of GPU resources and <0.6% latency-SLO violations "
                 "(4x H100 SXM 80GB)")


def cpu_baseline(w, objective: bool, factors=None, mixtures=False, seconds_target: float = 12.0):
    """The oracle, as it is, on a bounded slice of the first demand level."""
    import oracle
    pb, se = w.problems[0], w.searches[0]
    o = oracle.Oracle.from_problem(pb)
    if mixtures:
        o.set_mixtures(True)
    if objective:
        o.set_objective(1, 1.0, 0.035)
    threads = max(1, min(oracle.max_threads(), os.cpu_count() or 1))
    if factors is not None:
        # with per-variant factors the oracle searches whole levels: time the first few
        o.set_factors(factors)
        done, n_lv, t0 = 0, 0, time.perf_counter()
        for D in se.demand_mrps.tolist():
            res, _, _ = o.search([D], se.slo_latency_us, se.slo_accuracy, se.prune_cap, threads=threads)
            done += res[0].evaluated
            n_lv += 1
            if time.perf_counter() - t0 > seconds_target:
                break
        dt = time.perf_counter() - t0
        return {"value": done / dt, "unit": "candidates/s", "cores": threads, "kind": "oracle",
                "sample": f"the first {n_lv} demand levels of the same workload ({done} candidates), {dt:.1f} s"}
    D = int(se.demand_mrps[0])
    K, space, _ = o.space(D, se.slo_latency_us, se.prune_cap)

    def timed(nthreads, seconds):
        n = min(space, 1_000_000 * nthreads)       # probe for the rate, then a slice of the wanted length
        t0 = time.perf_counter()
        o.search_range(D, se.slo_latency_us, se.slo_accuracy, se.prune_cap, 0, n, threads=nthreads)
        rate = n / max(time.perf_counter() - t0, 1e-9)
        n2 = int(min(space, max(n, rate * seconds)))
        t0 = time.perf_counter()
        o.search_range(D, se.slo_latency_us, se.slo_accuracy, se.prune_cap, 0, n2, threads=nthreads)
        dt = time.perf_counter() - t0
        return n2, dt

    n1, dt1 = timed(1, seconds_target / 3)
    n2, dt = timed(threads, seconds_target)
    return {"value": n2 / dt, "unit": "candidates/s", "cores": threads, "kind": "oracle",
            "sample": f"first {n2} candidates of demand level 0 ({D} mrps) of the same workload, "
                      f"{dt:.1f} s",
            "all_threads": {"value": n2 / dt, "cores": threads},
            "single_thread": {"value": n1 / dt1, "cores": 1,
                              "sample": f"first {n1} candidates of the same level, {dt1:.1f} s"}}


def thinning_loss(jsv_mod, w, mixtures: bool):
    """What the prune cap costs (the thinning is a lossy rule of this library, not the paper's):
    the same sweep with the workload's cap and with a cap that never thins (single tuples: C; the
    exact front is then searched) - for mixtures, where no cap holds every option, cap 16 against
    cap 36 - and the per-level cost gap."""
    pb, se = w.problems[0], w.searches[0]
    j = jsv_mod.Jsv(device=0)
    if mixtures:
        j.set_mixtures(True)
    j.load(pb)
    lo_cap, hi_cap = (16, 36) if mixtures else (se.prune_cap, pb.C)
    a, sa = j.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, lo_cap)
    try:
        b, sb = j.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, hi_cap)
    except jsv_mod.JsvError:
        # the exact fronts of some level span more than a 63-bit key holds: twice the cap instead
        # (exact wherever no list is thinned at that cap; "reference_thinned" says where not)
        hi_cap = 2 * lo_cap
        b, sb = j.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, hi_cap)
    j.close()
    gaps = []
    for l, (x, y) in enumerate(zip(a, b)):
        gaps.append({"level": l, "demand_mrps": int(se.demand_mrps[l]),
                     "cost_capped": x.cost if x.feasible else None, "cost_reference": y.cost if y.feasible else None,
                     "thinned": bool(x.flags & 1), "reference_thinned": bool(y.flags & 1)})
    both = [(g["cost_capped"], g["cost_reference"]) for g in gaps if g["cost_capped"] is not None and g["cost_reference"] is not None]
    return {"cap": lo_cap, "reference_cap": hi_cap, "reference_is_exact_front": not any(g["reference_thinned"] for g in gaps),
            "levels_with_exact_reference": sum(not g["reference_thinned"] for g in gaps),
            "levels_feasible_capped": sum(g["cost_capped"] is not None for g in gaps),
            "levels_feasible_reference": sum(g["cost_reference"] is not None for g in gaps),
            "levels_costlier_when_capped": sum(x > y for x, y in both),
            "levels_cheaper_when_capped": sum(x < y for x, y in both),
            "max_relative_cost_gap": max([(x - y) / y for x, y in both], default=0.0),
            "candidates_capped": sum(r.evaluated for r in a), "candidates_reference": sum(r.evaluated for r in b),
            "ms_capped": sa.seconds_device * 1e3, "ms_reference": sb.seconds_device * 1e3,
            "max_demand_capped": sa.max_demand_mrps, "max_demand_reference": sb.max_demand_mrps,
            "per_level": gaps}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="xr8", choices=["chain3", "diamond5", "chain4", "xr8", "dagbatch", "traffic3"])
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run one 1 GiB device-to-device copy, a kernel of known HBM traffic "
                         "against which rocprofv3's FETCH_SIZE / WRITE_SIZE readings are scaled")
    ap.add_argument("--graph", action="store_true", help="replay the launch sequence as a HIP graph")
    ap.add_argument("--bounds", action="store_true",
                    help="time the library's default search, which skips what latency and capacity bounds "
                         "exclude in bulk, as the headline.  Without this flag the headline is the plain "
                         "enumeration (the tests of every candidate are issued) and the bounded search is "
                         "timed as a second leg, reported under with_bounds; results are the same")
    ap.add_argument("--prune-cap", type=int, default=None,
                    help="override the workload's per-task prune cap (single-system workloads)")
    ap.add_argument("--plain-only", action="store_true",
                    help="skip the second, bounded leg (for profiles of the plain enumeration alone)")
    ap.add_argument("--mixtures", action="store_true",
                    help="let a task run two tuples side by side (Eq. 9, 10); needs a pruned single-system workload")
    ap.add_argument("--no-peak-probe", action="store_true",
                    help="skip the microbenchmark of the vector ALUs' sustained issue rate")
    ap.add_argument("--peak-probe", action="store_true", help="(default) run that microbenchmark")
    ap.add_argument("--no-other-seeds", action="store_true",
                    help="default workload only: skip the one timed step each for seeds 1-3")
    ap.add_argument("--exact-front", action="store_true",
                    help="also report what the prune cap costs: the sweep at the workload's cap against a cap that "
                         "never thins (with --mixtures: cap 16 against cap 36), per-level cost gap")
    ap.add_argument("--objective", action="store_true",
                    help="maximise alpha*A_obj - beta*cost (alpha 1, beta 0.035) instead of minimum cost")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: the search runs on one GPU only; use --gpus 1")

    import torch
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    from paper_2603_08797_amd import jsv, workloads

    w = workloads.BENCH_WORKLOADS[args.workload](seed=args.seed)
    if args.prune_cap is not None:
        for se_ in w.searches:
            se_.prune_cap = args.prune_cap
        w.note += f", prune cap {args.prune_cap}"
    factors = w.meta.get("factor_milli")
    stream = torch.cuda.Stream(device=0)
    j = jsv.Jsv(device=0, stream=stream)
    if args.objective:
        j.set_objective(1, 1.0, 0.035)
    if args.graph:
        j.set_graph_mode(True)
    if args.mixtures:
        j.set_mixtures(True)
    j.set_bounds(args.bounds)
    batch = len(w.problems) > 1
    if batch:
        j.load_batch(w.problems, w.searches)
        n_levels = len(w.problems)
        j.lend_workspace(n_levels, 0)

        # (raw=True: the timed step hands back the C records as they are; turning them into
        # Python objects is the binding's convenience, not part of the search)
        def step():
            return j.search_loaded_batch(raw=True)
    else:
        pb, se = w.problems[0], w.searches[0]
        j.load(pb)
        if factors is not None:
            j.set_factors(factors)
        n_levels = len(se.demand_mrps)
        j.lend_workspace(n_levels, se.prune_cap)

        def step():
            return j.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap, raw=True)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    enum_s, dev_s, visited = [], [], 0
    for _ in range(args.steps):
        res, summ = step()
        enum_s.append(summ.seconds_enumerate)
        dev_s.append(summ.seconds_device)
        visited = summ.candidates_visited
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    res = j.results(res, batch)

    if args.copy_probe:
        src = torch.empty(1 << 30, dtype=torch.uint8, device="cuda")
        src.zero_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()

    with_bounds = None
    if not args.bounds and not args.plain_only:
        # second leg: the same steps with the bounds on (what a caller gets by default)
        j.set_bounds(True)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        for _ in range(args.steps):
            res_b, summ_b = step()
        torch.cuda.synchronize()
        wall_b = time.perf_counter() - t1
        res_b = j.results(res_b, batch)
        same = all((a.feasible, a.index, a.cost, a.choice) == (b.feasible, b.index, b.cost, b.choice)
                   for a, b in zip(res, res_b))
        with_bounds = {"ms_per_step": wall_b / args.steps * 1e3,
                       "ms_per_level": wall_b / args.steps * 1e3 / n_levels,
                       "enumerate_kernel_ms": summ_b.seconds_enumerate * 1e3,
                       "candidates_scored_per_step": min(summ_b.candidates_visited, sum(r.evaluated for r in res_b)),
                       "same_results_as_plain_enumeration": same}

    single_level = None
    if not batch and factors is None and n_levels > 1 and not args.graph and not args.plain_only and not args.bounds:
        # latency of one search over one demand level: the feasible level with the largest demand,
        # as a caller would ask for it (bounds on) and as the plain enumeration; 3 warm-up + 10 timed
        feas = [l for l, r in enumerate(res) if r.feasible]
        if feas:
            l1 = max(feas, key=lambda l: int(se.demand_mrps[l]))
            one = se.demand_mrps[l1:l1 + 1]
            single_level = {"level": l1, "demand_mrps": int(one[0]), "candidates": res[l1].evaluated}
            for name, on in (("with_bounds_ms", True), ("plain_ms", False)):
                j.set_bounds(on)
                for _ in range(3):
                    j.search(one, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
                torch.cuda.synchronize()
                t3 = time.perf_counter()
                for _ in range(10):
                    r1, _ = j.search(one, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
                torch.cuda.synchronize()
                single_level[name] = (time.perf_counter() - t3) / 10 * 1e3
                single_level["same_answer"] = single_level.get("same_answer", True) and \
                    (r1[0].feasible, r1[0].index, r1[0].cost) == (res[l1].feasible, res[l1].index, res[l1].cost)
            # the same for the feasible level with the smallest demand, whose optimum lies far below
            # S_avail (where the search with bounds starts from the plan kernel's first bound)
            l0 = min(feas, key=lambda l: int(se.demand_mrps[l]))
            if l0 != l1:
                low = {"level": l0, "demand_mrps": int(se.demand_mrps[l0])}
                one = se.demand_mrps[l0:l0 + 1]
                for name, on in (("with_bounds_ms", True), ("plain_ms", False)):
                    j.set_bounds(on)
                    for _ in range(3):
                        j.search(one, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
                    torch.cuda.synchronize()
                    t3 = time.perf_counter()
                    for _ in range(10):
                        r1, _ = j.search(one, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
                    torch.cuda.synchronize()
                    low[name] = (time.perf_counter() - t3) / 10 * 1e3
                    low["same_answer"] = low.get("same_answer", True) and \
                        (r1[0].feasible, r1[0].index, r1[0].cost) == (res[l0].feasible, res[l0].index, res[l0].cost)
                single_level["lowest_level"] = low
            j.set_bounds(args.bounds)

    other_seeds = None
    if (args.workload == "xr8" and not args.no_other_seeds and not batch and factors is None
            and not args.mixtures and not args.objective and not args.bounds and not args.graph):
        # the same configuration on the other seeds of the workload: one warm-up, one timed step each
        other_seeds = {}
        for sd in (1, 2, 3):
            if sd == args.seed:
                continue
            w2 = workloads.BENCH_WORKLOADS[args.workload](seed=sd)
            pb2, se2 = w2.problems[0], w2.searches[0]
            cap2 = args.prune_cap if args.prune_cap is not None else se2.prune_cap
            j.set_bounds(False)
            j.load(pb2)
            j.search(se2.demand_mrps, se2.slo_latency_us, se2.slo_accuracy, cap2)
            torch.cuda.synchronize()
            t2 = time.perf_counter()
            r2, s2 = j.search(se2.demand_mrps, se2.slo_latency_us, se2.slo_accuracy, cap2)
            torch.cuda.synchronize()
            dt2 = time.perf_counter() - t2
            n2 = sum(r.evaluated for r in r2)
            other_seeds[str(sd)] = {"candidates_per_step": n2, "ms_per_step": dt2 * 1e3, "candidates_per_s": n2 / dt2,
                                    "enumerate_kernel_ms": s2.seconds_enumerate * 1e3,
                                    "feasible_levels": sum(1 for r in r2 if r.feasible),
                                    "max_serviceable_demand_mrps": s2.max_demand_mrps}

    candidates = sum(r.evaluated for r in res)
    ms_per_step = wall / args.steps * 1e3
    enum_avg = sum(enum_s) / len(enum_s) or sum(dev_s) / len(dev_s)     # graph mode times the whole replay
    # The roofline counts the candidates whose tests the kernel issued; with bounds on, the rest
    # of the searched space was excluded in bulk and costs (almost) nothing.
    scored = min(visited, candidates)
    ops = algorithmic_ops(res, args.mixtures) * scored / max(candidates, 1)
    achieved = ops / enum_avg
    ops_prev = previous_rule_ops(jsv, w.problems, w.searches, res, factors, args.mixtures)
    if ops_prev is not None:
        ops_prev *= scored / max(candidates, 1)
    out = {
        "metric": "candidate assignments evaluated/sec on 1 MI355X; ms to optimum per demand level",
        "value": candidates / (wall / args.steps),
        "unit": "candidates/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "ms_per_level": ms_per_step / n_levels,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "u32+f64", "data": "synthetic",
        "config": {"workload": f"{w.name} seed {args.seed}: {w.note}", "levels_or_problems": n_levels,
                   "objective": "alpha*A_obj - beta*cost, alpha 1, beta 0.035" if args.objective else "minimum cost",
                   "mixtures": bool(args.mixtures),
                   "candidates_per_step": candidates,
                   "bounds": bool(args.bounds),
                   "candidates_scored_per_step": scored,
                   "scored_per_s": scored / (wall / args.steps),
                   "feasible_levels": sum(1 for r in res if r.feasible),
                   "max_serviceable_demand_mrps": summ.max_demand_mrps},
        "roofline": {"bound": "alu", "achieved": achieved / 1e12, "peak": VALU_PEAK_LANE_OPS / 1e12,
                     "unit": "Tlane-op/s", "frac": achieved / VALU_PEAK_LANE_OPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, args.seed, args.objective, args.mixtures, bool(args.bounds))),
                     "kernel": "enumerate_kernel", "kernel_ms": enum_avg * 1e3,
                     "ops_per_candidate": (ops or 0.0) / max(scored, 1),
                     "previous_rule": None if ops_prev is None else {
                         "ops_per_candidate": ops_prev / max(scored, 1),
                         "frac": ops_prev / enum_avg / VALU_PEAK_LANE_OPS},
                     "unshared_count": {"ops_per_candidate": UNSHARED_OPS_PER_CANDIDATE,
                                        "frac": UNSHARED_OPS_PER_CANDIDATE * scored / enum_avg / VALU_PEAK_LANE_OPS},
                     "device_ms_all_kernels": sum(dev_s) / len(dev_s) * 1e3},
        "context": PAPER_CONTEXT,
    }
    key = (args.workload, args.seed, args.objective, args.mixtures, bool(args.bounds))
    if key in MEASURED_COUNTERS and args.prune_cap is None:
        out["roofline"]["counters"] = MEASURED_COUNTERS[key]
    if not args.no_peak_probe:
        probe = peak_probe()
        out["roofline"]["peak_measured"] = probe
        if probe and probe.get("v_min_u32"):
            # against the issue rate of the loop's own instructions (compare and minimum)
            out["roofline"]["frac_of_measured_peak"] = achieved / (probe["v_min_u32"] * 1e12)
    if single_level is not None:
        out["single_level"] = single_level
    if other_seeds is not None:
        out["config"]["other_seeds"] = other_seeds
    if with_bounds is not None:
        out["with_bounds"] = with_bounds
    if args.exact_front and not batch and factors is None:
        out["thinning_loss"] = thinning_loss(jsv, w, args.mixtures)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w, args.objective, factors, args.mixtures)
    j.close()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
