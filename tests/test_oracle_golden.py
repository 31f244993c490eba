"""Pin 1: the hand-worked two-task chain (tests/golden/p1_two_task_chain.json)."""
import json
import os

import numpy as np
import pytest

import oracle

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def g():
    with open(os.path.join(HERE, "golden", "p1_two_task_chain.json")) as f:
        return json.load(f)


def make(g, capacity=0, thr=None):
    lat = np.array(g["latency_us"], dtype=np.uint32).reshape(g["T"], g["V"], g["P"], g["B"])
    acc = np.array(g["accuracy"], dtype=np.float64)
    src = [e[0] for e in g["edges"]]
    dst = [e[1] for e in g["edges"]]
    return oracle.Oracle(g["T"], g["V"], g["P"], g["B"], g["units"], g["batch"], lat, thr, acc,
                         src, dst, g["mult_milli"], capacity, g["queue_factor"])


def test_amax_and_single_path(g):
    o = make(g)
    assert o.amax() == pytest.approx(g["amax"], rel=1e-15)
    assert o.paths() == [([0, 1], 1.0)]


def test_derived_throughput_matches_explicit_table(g):
    thr = np.array(g["derived_thr_mrps"], dtype=np.uint32).reshape(2, 2, 2, 2)
    a, b = make(g), make(g, thr=thr)
    for o in (a, b):
        rep, cost = o.cost_table(g["at_260_rps"]["demand_mrps"])
        assert rep.tolist() == g["at_260_rps"]["replicas"]
        assert cost.tolist() == g["at_260_rps"]["cost"]


def test_three_searches_at_260_rps(g):
    o = make(g)
    D = g["at_260_rps"]["demand_mrps"]
    for s in g["at_260_rps"]["searches"]:
        res, bl, md = o.search([D], s["slo_latency_us"], s["slo_accuracy"], 0)
        r = res[0]
        assert r.feasible and bl == 0 and md == D
        assert r.index == s["index"] and r.full_index == s["index"]
        assert r.choice == s["choice"]
        assert r.cost == s["cost"]
        assert r.latency_us == s["latency_us"]
        assert r.accuracy == pytest.approx(s["accuracy_num"] / s["accuracy_den"], rel=1e-14)
        assert r.evaluated == 64 and r.flags == 0
        assert r.replicas == [g["at_260_rps"]["replicas"][t][r.choice[t]] for t in range(2)]


def test_sweep_and_max_serviceable_demand(g):
    sw = g["sweep"]
    o = make(g, capacity=sw["capacity_units"])
    res, bl, md = o.search(sw["demand_mrps"], sw["slo_latency_us"], sw["slo_accuracy"], 0)
    for r, idx, cost in zip(res, sw["index"], sw["cost"]):
        if idx is None:
            assert not r.feasible and r.index == 2**64 - 1 and r.cost == 2**31 - 1
        else:
            assert r.feasible and r.index == idx and r.cost == cost
    assert bl == sw["best_level"] and md == sw["max_demand_mrps"]
    o = make(g, capacity=0)
    res, bl, md = o.search(sw["demand_mrps"], sw["slo_latency_us"], sw["slo_accuracy"], 0)
    assert [r.cost for r in res] == sw["unlimited_capacity_cost"]
    assert [r.index for r in res] == [48] * 5
    assert bl == 4 and md == 800000


def test_sweep_order_does_not_matter(g):
    sw = g["sweep"]
    o = make(g, capacity=sw["capacity_units"])
    d = [800000, 260000, 400000, 100000, 200000]
    res, bl, md = o.search(d, sw["slo_latency_us"], sw["slo_accuracy"], 0)
    assert [r.feasible for r in res] == [False, True, True, True, True]
    assert bl == 2 and md == 400000


def test_accuracy_feasible_variant_pairs(g):
    o = make(g)
    ok = [[va, vb] for va in range(2) for vb in range(2)
          if o.accuracy_of_variants([va, vb]) >= 0.85]
    assert ok == g["accuracy_feasible_variant_pairs_at_0.85"]
    assert o.accuracy_of_variants([1, 1]) == pytest.approx(1.0, rel=1e-15)


def test_eval_matches_table(g):
    o = make(g)
    D = g["at_260_rps"]["demand_mrps"]
    idx = np.arange(64, dtype=np.uint64)
    lat, rep, cost, acc, mask = o.eval(D, 40000, 0.85, 0, idx)
    L = g["latency_us"]
    K = g["at_260_rps"]["cost"]
    A = g["accuracy"]
    for i in range(64):
        ca, cb = i % 8, i // 8
        assert lat[i] == 2 * (L[0][ca] + L[1][cb])
        assert cost[i] == K[0][ca] + K[1][cb]
        a = A[0][ca // 4] * A[1][cb // 4] / 0.855
        assert acc[i] == pytest.approx(a, rel=1e-14)
        assert mask[i] == (1 if lat[i] <= 40000 else 0) | (2 if a >= 0.85 else 0) | 4
