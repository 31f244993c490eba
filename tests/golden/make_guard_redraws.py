"""Writes paper_2603_08797_amd/guard_redraws.json.

The benchmark inputs must keep every candidate's accuracy more than 1e-9 away
from the accuracy SLO, so that the feasibility mask is the same whichever
order the fp64 products are taken in.  Accuracy depends only on the variants,
so the CPU oracle checks all V^T variant combinations; where the first draw
fails, the accuracy table (for the batch workload: the accuracy SLO) is drawn
again and the number of redraws is recorded.  Calls the oracle only.

Run from the repository root:  python tests/golden/make_guard_redraws.py
"""
import json
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

import oracle  # noqa: E402
from paper_2603_08797_amd import workloads as W  # noqa: E402

BAND = 1e-9
CASES = [("chain3", [0]), ("diamond5", [0]), ("chain4", [0]), ("xr8", [0, 1, 2, 3]), ("traffic3", [0])]


def margin(pb, se):
    return oracle.Oracle.from_problem(pb).accuracy_margin(se.slo_accuracy)


def main():
    table = {}
    for name, seeds in CASES:
        for seed in seeds:
            for redraw in range(100):
                w = W.BENCH_WORKLOADS[name](seed=seed, redraw=redraw)
                if margin(w.problems[0], w.searches[0]) > BAND:
                    break
            else:
                raise SystemExit(f"{name} seed {seed}: no draw clears the band")
            if redraw:
                table[f"{name}/seed{seed}/0"] = redraw
    # batch workload: redraw only the accuracy SLO of the offending problem
    seed = 0
    w = W.dagbatch(seed=seed)
    for k, (pb, se) in enumerate(zip(w.problems, w.searches)):
        o = oracle.Oracle.from_problem(pb)
        redraw = 0
        slo = se.slo_accuracy
        while o.accuracy_margin(slo) <= BAND:
            redraw += 1
            slo = 0.3 + 0.4 * W.SplitMix64(5, seed, 5, k, redraw).uniform()
        if redraw:
            table[f"dagbatch/seed{seed}/{k}"] = redraw
    out = os.path.join(ROOT, "paper_2603_08797_amd", "guard_redraws.json")
    with open(out, "w") as f:
        json.dump(table, f, indent=1, sort_keys=True)
        f.write("\n")
    print(f"wrote {out}: {table}")


if __name__ == "__main__":
    main()
