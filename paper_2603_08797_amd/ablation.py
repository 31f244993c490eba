"""Maximum serviceable demand of the eight A / S / T search spaces (the analysis of
Fig. 3 of the paper) on a synthetic traffic-analysis-like system: a detector feeding two
classifiers, one of them invoked twice per detection, on a testbed of 840 partition units.

    python -m paper_2603_08797_amd.ablation [--seed N]

One jsv_search call per search space sweeps 160 log-spaced demand levels; the ratios are
relative to the unoptimised space (no accuracy scaling, whole GPUs, static budgets).  The
numbers depend on the synthetic profile tables and are not comparable with the paper's.
"""
from __future__ import annotations

import argparse
import itertools

import numpy as np

from . import jsv, workloads


def system(seed: int):
    pb = workloads.diamond5(seed=seed).problems[0]
    T = 3
    return workloads.Problem(T, pb.V, pb.P, pb.B, pb.units, pb.batch, pb.latency_us[:T].copy(),
                             pb.thr_mrps[:T].copy(), pb.accuracy[:T].copy(),
                             np.array([0, 0], dtype=np.uint16), np.array([1, 2], dtype=np.uint16),
                             np.array([1000, 2000, 1000], dtype=np.uint32), 840, 2)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--slo-latency-ms", type=float, default=120.0)
    ap.add_argument("--slo-accuracy", type=float, default=0.9)
    args = ap.parse_args()
    pb = system(args.seed)
    demand = np.unique(np.round(1000 * 2.0 * 1.06 ** np.arange(160)).astype(np.uint32))
    j = jsv.Jsv(device=0)
    rows = []
    for a, s, t in itertools.product([False, True], repeat=3):
        j.set_search_space(a, s, t)
        j.load(pb)
        res, summ = j.search(demand, int(args.slo_latency_ms * 1000), args.slo_accuracy, 0)
        used = res[summ.best_level].cost if summ.best_level >= 0 else 0
        name = "+".join(n for n, on in zip("AST", (a, s, t)) if on) or "Unopt"
        rows.append((name, summ.max_demand_mrps / 1000.0, used, summ.seconds_device * 1e3))
    j.close()
    base = rows[0][1] or float("nan")
    print(f"{'space':8} {'max rps':>10} {'x Unopt':>8} {'units used':>11} {'device ms':>10}")
    for name, rps, used, ms in rows:
        print(f"{name:8} {rps:10.1f} {rps / base:8.2f} {used:7d}/840 {ms:10.3f}")


if __name__ == "__main__":
    main()
