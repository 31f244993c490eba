"""Pins of the oracle's Eq. 14 mode (maximise alpha*A_obj - beta*cost)."""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2603_08797_amd import workloads as W
from pyref import PyRef

HERE = os.path.dirname(os.path.abspath(__file__))
U32 = 2**32 - 1


def test_hand_worked_chain_objective():
    with open(os.path.join(HERE, "golden", "p1_two_task_chain.json")) as f:
        g = json.load(f)
    e = g["objective_eq14"]
    lat = np.array(g["latency_us"], dtype=np.uint32).reshape(2, 2, 2, 2)
    o = oracle.Oracle(2, 2, 2, 2, g["units"], g["batch"], lat, None, np.array(g["accuracy"]),
                      [0], [1], g["mult_milli"], 0, 2)
    o.set_objective(1, e["alpha"], e["beta"])
    r = o.search([e["demand_mrps"]], e["slo_latency_us"], e["slo_accuracy"], 0)[0][0]
    assert (r.index, r.choice, r.cost, r.latency_us) == (e["index"], e["choice"], e["cost"], e["latency_us"])
    assert r.accuracy == pytest.approx(e["accuracy"], rel=1e-15)
    assert r.objective == pytest.approx(e["objective"], rel=1e-13)
    gap = o.objective_margin(e["demand_mrps"], e["slo_latency_us"], e["slo_accuracy"], 0)
    want = e["objective"] - (e["runner_up_objective_num"] / e["runner_up_objective_den"] - e["beta"] * e["runner_up_cost"])
    assert gap == pytest.approx(want, rel=1e-12)


@pytest.mark.parametrize("seed", range(120))
def test_tiny_random_against_exact_rationals(seed):
    pb, se = W.tiny_random(seed + 900)
    o = oracle.Oracle.from_problem(pb)
    ref = PyRef(pb)
    r0 = W.SplitMix64(91, seed)
    alpha, beta = [(1.0, 0.035), (1.0, 0.002), (0.3, 0.05), (2.0, 0.0)][r0.randint(0, 3)]
    o.set_objective(1, alpha, beta)
    for D in se.demand_mrps.tolist():
        best, gap = ref.search_objective(D, se.slo_latency_us, se.slo_accuracy, se.prune_cap, alpha, beta)
        base, K, _, margin = ref.search(D, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
        if margin is not None and margin <= 1e-9:
            continue                                   # accuracy SLO guard band
        r = o.search([D], se.slo_latency_us, se.slo_accuracy, se.prune_cap)[0][0]
        if best is None:
            assert not r.feasible
            continue
        if gap is not None and gap <= 1e-9:
            continue                                   # objective guard band
        idx, cost, lat, acc, choice, obj = best
        assert r.feasible and (r.index, r.cost, r.latency_us, r.choice) == (idx, cost, lat, choice)
        assert r.objective == pytest.approx(float(obj), rel=1e-12, abs=1e-13)
        m = o.objective_margin(D, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
        assert m == (1e300 if gap is None else pytest.approx(float(gap), rel=1e-9, abs=1e-12))


@pytest.mark.parametrize("seed", range(25))
def test_alpha_zero_is_the_cheapest_feasible_assignment(seed):
    pb, se = W.tiny_random(seed + 1000, T=3)
    a, b = oracle.Oracle.from_problem(pb), oracle.Oracle.from_problem(pb)
    b.set_objective(1, 0.0, 0.035)
    for D in se.demand_mrps.tolist():
        ra = a.search([D], se.slo_latency_us, se.slo_accuracy, 0)[0][0]
        rb = b.search([D], se.slo_latency_us, se.slo_accuracy, 0)[0][0]
        assert (ra.feasible, ra.index, ra.cost) == (rb.feasible, rb.index, rb.cost)


@pytest.mark.parametrize("seed", range(25))
def test_beta_zero_maximises_accuracy_then_cost(seed):
    pb, se = W.tiny_random(seed + 1100, T=3)
    pb.capacity_units = 0
    o = oracle.Oracle.from_problem(pb)
    o.set_objective(1, 1.0, 0.0)
    D = int(se.demand_mrps[0])
    r = o.search([D], se.slo_latency_us, 0.0, 0)[0][0]
    K, space, _ = o.space(D, se.slo_latency_us, 0)
    lat, rep, cost, acc, mask = o.eval(D, se.slo_latency_us, 0.0, 0, np.arange(space, dtype=np.uint64))
    ok = mask == 7
    if not ok.any():
        assert not r.feasible
        return
    top = acc[ok].max()
    tied = [(int(cost[i]), i) for i in range(space) if ok[i] and acc[i] == top]
    assert (r.cost, r.index) == min(tied) and r.accuracy == top


def test_objective_never_below_the_cheapest_assignments_objective():
    w = W.chain3()
    pb, se = w.problems[0], w.searches[0]
    a, b = oracle.Oracle.from_problem(pb), oracle.Oracle.from_problem(pb)
    b.set_objective(1, 1.0, 0.035)
    ra = a.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0, threads=4)[0][0]
    rb = b.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0, threads=4)[0][0]
    assert rb.objective >= ra.objective and rb.cost >= ra.cost and rb.accuracy >= ra.accuracy
    assert b.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0, threads=1)[0][0] == rb


def test_bad_objective_arguments():
    pb, _ = W.tiny_random(1, T=2)
    o = oracle.Oracle.from_problem(pb)
    for args in [(2, 1.0, 0.035), (1, -1.0, 0.035), (1, 1.0, float("nan"))]:
        with pytest.raises(oracle.OracleError):
            o.set_objective(*args)
