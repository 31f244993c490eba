"""Pins for the parts of the oracle that the other oracle tests take on trust.

Hand-worked lists (tests/golden/p2_thinning_and_budgets.json) for the two thinning rules of
the prune and for the static budgets of Appendix B; exact-rational values (tests/pyref.py)
for the three guard-band helpers - orc_accuracy_margin, orc_mixture_margin,
orc_budget_margin - which decide what the parity tests and the input generators skip.
"""
import json
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2603_08797_amd import workloads as W
from pyref import PyRef

HERE = os.path.dirname(os.path.abspath(__file__))
with open(os.path.join(HERE, "golden", "p2_thinning_and_budgets.json")) as f:
    G = json.load(f)
with open(os.path.join(HERE, "golden", "p1_two_task_chain.json")) as f:
    P1 = json.load(f)


def _single_task_oracle(g, latency, capacity=0):
    T, V, P, B = g["T"], g["V"], g["P"], g["B"]
    lat = np.array(latency, dtype=np.uint32).reshape(T, V, P, B)
    thr = np.full((T, V, P, B), g["thr_mrps_all"], dtype=np.uint32)
    return oracle.Oracle(T, V, P, B, g["units"], g["batch"], lat, thr, np.array(g["accuracy"]), [], [], [1000],
                         capacity, 2)


# ---- thinning of single tuples (prune step c) ----------------------------------------------
@pytest.mark.parametrize("case", ["case_a", "case_b"])
def test_hand_worked_thinning_of_single_tuples(case):
    g = G["thinning_single_tuples"]
    o = _single_task_oracle(g, g[case]["latency_us"])
    # the exact front first: a cap no smaller than it thins nothing
    ids, tr = o.pruned(g["demand_mrps"], g["slo_latency_us"], g["V"] * g["P"] * g["B"], 0)
    assert ids.tolist() == g[case]["front"] and not tr
    for c in g[case]["caps"]:
        ids, tr = o.pruned(g["demand_mrps"], g["slo_latency_us"], c["cap"], 0)
        assert ids.tolist() == c["kept"], c
        assert int(tr) == c["truncated"], c


def test_a_planted_rank_mistake_would_fail_the_thinning_fixture():
    """The fixture tells floor from round and (n-1)/(quota-1) from n/quota: the ranks those
    variants would keep differ from the expected lists."""
    order = [0, 1, 2, 3, 4, 6]                      # case b, variant 0 in latency order
    n, quota = 6, 3
    right = [order[(j * (n - 1)) // (quota - 1)] for j in range(quota)]
    rounded = [order[int(j * (n - 1) / (quota - 1) + 0.5)] for j in range(quota)]
    strided = [order[(j * n) // quota] for j in range(quota)]
    want = [k for k in G["thinning_single_tuples"]["case_b"]["caps"][0]["kept"] if k < 7]
    assert right == want and rounded != want and strided != want


# ---- thinning of options (mixture mode, prune step c) --------------------------------------
def test_hand_worked_thinning_of_options():
    g = G["thinning_options"]
    o = _single_task_oracle(g, g["latency_us"], capacity=g["capacity_units"])
    o.set_mixtures(True)
    units = g["units"]
    for c in g["caps"]:
        opts, tr = o.options(g["demand_mrps"], g["slo_latency_us"], c["cap"], 0)
        assert [x[0] for x in opts] == c["kept"], c
        assert int(tr) == c["truncated"], c
        for c1, c2, m1, m2, lat, cost, acc in opts:         # single tuples, one replica each
            assert (c2, m1, m2) == (0xFFFF, 1, 0)
            assert lat == np.array(g["latency_us"]).ravel()[c1] and cost == units[c1 % 3]
            assert acc == g["accuracy"][0][c1 // 3]


# ---- static budgets of Appendix B -----------------------------------------------------------
def _p1_oracle(capacity):
    lat = np.array(P1["latency_us"], dtype=np.uint32).reshape(2, 2, 2, 2)
    return oracle.Oracle(2, 2, 2, 2, P1["units"], P1["batch"], lat, None, np.array(P1["accuracy"]), [0], [1],
                         P1["mult_milli"], capacity, 2)


def test_hand_worked_static_budgets():
    b = G["appendix_b_budgets"]
    o = _p1_oracle(b["capacity_units"])
    o.set_search_space(True, True, False)
    for t in range(2):
        ids, _ = o.pruned(b["demand_mrps"], b["slo_latency_us"], 0, t)
        assert ids.tolist() == b["allowed"][t]
    s = b["search"]
    res, _, _ = o.search([b["demand_mrps"]], b["slo_latency_us"], s["slo_accuracy"], 0)
    r = res[0]
    assert (r.feasible, r.index, r.full_index, r.choice, r.cost, r.latency_us) == \
           (True, s["index"], s["full_index"], s["choice"], s["cost"], s["latency_us"])
    assert abs(r.accuracy - s["accuracy_num"] / s["accuracy_den"]) < 1e-14
    # the budgets themselves: the margin helper sees the same shares
    frac = [x - int(x) for x in b["unit_shares"]]
    assert abs(o.budget_margin() - min(min(f, 1 - f) for f in frac)) < 1e-5
    # the budgets bite: with graph-informed (end-to-end) constraints ids 5 and 6 are back
    o.set_search_space(True, True, True)
    ids, _ = o.pruned(b["demand_mrps"], b["slo_latency_us"], 0, 0)
    assert ids.tolist() == list(range(8))


def test_static_budgets_with_one_partition_only():
    """S off as well: the reference tuple is taken over the whole-GPU partition only (ids 6, 7 of
    the most accurate variant).  A: reference latency 20000, best throughput 100000 at 2 units;
    B: 15000 and 133333 at 2 units.  Latency: A 2*L*35000 <= 70000*20000 -> L <= 20000,
    B L <= 15000; shares as before (6 and 5 units).  Allowed, among the 2-unit choices
    2, 3, 6, 7: A latencies 6000, 10000, 12000, 20000 and costs 4, 4, 8, 6 -> 2, 3, 7;
    B latencies 3000, 5000, 9000, 15000 and costs 2, 2, 6, 4 -> 2, 3, 7."""
    b = G["appendix_b_budgets"]
    o = _p1_oracle(b["capacity_units"])
    o.set_search_space(True, False, False)
    for t in range(2):
        ids, _ = o.pruned(b["demand_mrps"], b["slo_latency_us"], 0, t)
        assert ids.tolist() == [2, 3, 7]


# ---- guard-band helpers against exact rationals -----------------------------------------------
@pytest.mark.parametrize("seed", range(60))
def test_accuracy_margin_is_the_exact_minimum_distance(seed):
    pb, se = W.tiny_random(seed + 4000)
    o = oracle.Oracle.from_problem(pb)
    ref = PyRef(pb)
    import itertools
    for slo in (se.slo_accuracy, 0.5, 0.8123, 1.0):
        want = min(abs(ref._acc(vs) / ref.amax - Fraction(float(slo)))
                   for vs in itertools.product(range(pb.V), repeat=pb.T))
        assert abs(o.accuracy_margin(slo) - float(want)) <= 1e-14


def test_accuracy_margin_on_the_hand_worked_chain():
    """A_obj of the four variant pairs: 0.56, 0.76, 0.63, 0.855 over 0.855.  At SLO_a = 0.85 the
    nearest is 0.76/0.855 = 0.88889 (distance 0.03889); at 0.74 it is 0.63/0.855 = 0.73684."""
    o = _p1_oracle(0)
    assert abs(o.accuracy_margin(0.85) - (0.76 / 0.855 - 0.85)) < 1e-15
    assert abs(o.accuracy_margin(0.74) - (0.74 - 0.63 / 0.855)) < 1e-15
    assert o.accuracy_margin(1.0) == 0.0


@pytest.mark.parametrize("seed", range(40))
def test_mixture_margin_is_the_exact_minimum_distance(seed):
    pb, se = W.tiny_mixture(5000 + seed)
    import dataclasses
    if pb.capacity_units == 0:
        pb = dataclasses.replace(pb, capacity_units=30)
    cap = [4, 7, 12, 40][seed % 4]
    o = oracle.Oracle.from_problem(pb)
    o.set_mixtures(True)
    ref = PyRef(pb)
    D = int(se.demand_mrps[0])
    try:
        best, K, tr, margin = ref.search_mix(D, se.slo_latency_us, se.slo_accuracy, cap, max_space=60000)
    except OverflowError:
        pytest.skip("space too large for the exact reference")
    got = o.mixture_margin(D, se.slo_latency_us, se.slo_accuracy, cap)
    if margin is None:
        assert got == 1e300
    else:
        assert abs(got - float(margin)) <= 1e-13


@pytest.mark.parametrize("seed", range(60))
def test_budget_margin_is_the_exact_distance_to_a_whole_share(seed):
    pb, se = W.tiny_random(seed + 4100)
    import dataclasses
    if pb.capacity_units == 0:
        pb = dataclasses.replace(pb, capacity_units=17 + seed)
    o = oracle.Oracle.from_problem(pb)
    assert o.budget_margin() == 0.5                     # no static budgets: nothing to guard
    for spatial in (True, False):
        o.set_search_space(True, spatial, False)
        ref = PyRef(pb)
        ref.space = (True, spatial, False)
        shares = ref.resource_shares()
        want = min(min(s - (s.numerator // s.denominator), 1 - (s - (s.numerator // s.denominator)))
                   for s in shares)
        assert abs(o.budget_margin() - float(want)) <= 1e-9
