"""The hand-worked thinning and budget examples (tests/golden/p2_thinning_and_budgets.json) on the GPU."""
import json
import os

import numpy as np
import pytest

from paper_2603_08797_amd import jsv

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))
with open(os.path.join(HERE, "golden", "p2_thinning_and_budgets.json")) as f:
    G = json.load(f)
with open(os.path.join(HERE, "golden", "p1_two_task_chain.json")) as f:
    P1 = json.load(f)


@pytest.fixture(scope="module")
def ctx():
    j = jsv.Jsv(device=0)
    yield j
    j.close()


@pytest.mark.parametrize("case", ["case_a", "case_b"])
def test_hand_worked_thinning_of_single_tuples(ctx, case):
    g = G["thinning_single_tuples"]
    T, V, P, B = g["T"], g["V"], g["P"], g["B"]
    lat = np.array(g[case]["latency_us"], dtype=np.uint32).reshape(T, V, P, B)
    thr = np.full((T, V, P, B), g["thr_mrps_all"], dtype=np.uint32)
    ctx.load_profile(T, V, P, B, g["units"], g["batch"], lat, thr, np.array(g["accuracy"]))
    ctx.set_dag(T, [], [], [1000], 0, 2)
    ids, tr = ctx.get_pruned(g["demand_mrps"], g["slo_latency_us"], V * P * B, 0)
    assert ids.tolist() == g[case]["front"] and not tr
    for c in g[case]["caps"]:
        ids, tr = ctx.get_pruned(g["demand_mrps"], g["slo_latency_us"], c["cap"], 0)
        assert ids.tolist() == c["kept"] and int(tr) == c["truncated"], c


def test_hand_worked_thinning_of_options():
    """Mixture mode has no list read-out; the thinned lists show in what a search can still
    find.  With SLO_a = 0 and no latency limit the cheapest option wins (id 2: 1 unit, kept by
    every cap); with the accuracy of variant 2 demanded, the cheapest kept option of that variant:
    id 8 (1 unit) at every cap; with a latency SLO of 2*2800 the latency filter leaves six options
    (ids 0, 3, 6, 1, 4, 7), thinned only at cap 4, and id 7 (2 units) is the cheapest of variant 2."""
    g = G["thinning_options"]
    T, V, P, B = g["T"], g["V"], g["P"], g["B"]
    lat = np.array(g["latency_us"], dtype=np.uint32).reshape(T, V, P, B)
    thr = np.full((T, V, P, B), g["thr_mrps_all"], dtype=np.uint32)
    j = jsv.Jsv(device=0)
    try:
        j.set_mixtures(True)
        j.load_profile(T, V, P, B, g["units"], g["batch"], lat, thr, np.array(g["accuracy"]))
        j.set_dag(T, [], [], [1000], g["capacity_units"], 2)
        for c in g["caps"]:
            r = j.search([g["demand_mrps"]], g["slo_latency_us"], 0.0, c["cap"])[0][0]
            assert (r.choice, r.cost, r.evaluated, r.flags & 1) == ([2], 1, len(c["kept"]), c["truncated"]), c
            r = j.search([g["demand_mrps"]], g["slo_latency_us"], 0.95, c["cap"])[0][0]
            assert (r.choice, r.cost) == ([8], 1), c
            # the latency filter runs before the thinning: with 5600 us only ids 0,3,6,1,4,7
            # (latency <= 2800) enter it, 6 options
            r = j.search([g["demand_mrps"]], 5600, 0.95, c["cap"])[0][0]
            if c["cap"] >= 6:
                assert (r.choice, r.cost, r.flags & 1) == ([7], 2, 0), c
            else:
                # cap 4: bands 2, per 2 over 0, 3, 6 | 1, 4, 7: band 0 by accuracy 0, 3, 6 keeps 0, 6;
                # band 1 keeps 1, 7 -> id 7 is still there
                assert (r.choice, r.cost, r.flags & 1, r.evaluated) == ([7], 2, 1, 4), c
    finally:
        j.close()


def test_hand_worked_static_budgets(ctx):
    b = G["appendix_b_budgets"]
    lat = np.array(P1["latency_us"], dtype=np.uint32).reshape(2, 2, 2, 2)
    ctx.load_profile(2, 2, 2, 2, P1["units"], P1["batch"], lat, None, np.array(P1["accuracy"]))
    ctx.set_dag(2, [0], [1], P1["mult_milli"], b["capacity_units"], 2)
    ctx.set_search_space(True, True, False)
    try:
        for t in range(2):
            ids, _ = ctx.get_pruned(b["demand_mrps"], b["slo_latency_us"], 0, t)
            assert ids.tolist() == b["allowed"][t]
        s = b["search"]
        r = ctx.search([b["demand_mrps"]], b["slo_latency_us"], s["slo_accuracy"], 0)[0][0]
        assert (r.feasible, r.index, r.full_index, r.choice, r.cost, r.latency_us) == \
               (True, s["index"], s["full_index"], s["choice"], s["cost"], s["latency_us"])
        assert abs(r.accuracy - s["accuracy_num"] / s["accuracy_den"]) < 1e-14
        ctx.set_search_space(True, False, False)
        for t in range(2):
            ids, _ = ctx.get_pruned(b["demand_mrps"], b["slo_latency_us"], 0, t)
            assert ids.tolist() == [2, 3, 7]
    finally:
        ctx.set_search_space(True, True, True)
