"""Pins of the oracle's two-tuple mixtures (Eq. 2, 6, 7, 9, 10): hand-worked options and search,
an independent brute force, reductions to the single-tuple search, invariants."""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2603_08797_amd import workloads
from pyref import PyRef

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def g():
    with open(os.path.join(HERE, "golden", "p1_two_task_chain.json")) as f:
        return json.load(f)


def make(g, capacity=0):
    lat = np.array(g["latency_us"], dtype=np.uint32).reshape(g["T"], g["V"], g["P"], g["B"])
    acc = np.array(g["accuracy"], dtype=np.float64)
    o = oracle.Oracle(g["T"], g["V"], g["P"], g["B"], g["units"], g["batch"], lat, None, acc,
                      [e[0] for e in g["edges"]], [e[1] for e in g["edges"]], g["mult_milli"], capacity,
                      g["queue_factor"])
    o.set_mixtures(True)
    return o


def test_hand_worked_options(g):
    mx = g["mixtures_eq9_10"]
    o = make(g)
    opts, tr = o.options(mx["demand_mrps"], 100000, 0, mx["task"])
    assert not tr
    # single tuples first, as in the fixed-factor tables
    single = [x for x in opts if x[1] == 0xFFFF]
    assert [x[0] for x in single] == list(range(8))
    assert [x[2] for x in single] == g["at_260_rps"]["replicas"][0]
    assert [x[5] for x in single] == g["at_260_rps"]["cost"][0]
    ids = [x[0] if x[1] == 0xFFFF else 8 + (x[0] * 8 + x[1]) * 65536 + x[2] for x in opts]
    assert ids == sorted(ids) and len(set(ids)) == len(ids)
    for pair in mx["pairs"]:
        got = [x for x in opts if (x[0], x[1]) == (pair["c1"], pair["c2"])]
        assert [(x[2], x[3], x[5], x[4]) for x in got] == \
               [(w["m1"], w["m2"], w["cost"], w["latency_us"]) for w in pair["options"]]
        for x, w in zip(got, pair["options"]):
            assert x[6] == pytest.approx(w["acc_num"] / w["acc_den"], rel=1e-15)


def test_hand_worked_search(g):
    s = g["mixtures_eq9_10"]["search"]
    o = make(g)
    r = o.search([g["mixtures_eq9_10"]["demand_mrps"]], s["slo_latency_us"], s["slo_accuracy"], 0)[0][0]
    assert r.feasible and r.cost == s["cost"] and r.latency_us == s["latency_us"]
    assert (r.choice, r.choice2, r.replicas, r.replicas2) == (s["choice"], s["choice2"], s["replicas"], s["replicas2"])
    assert r.accuracy == pytest.approx(s["accuracy_num"] / s["accuracy_den"] * s["accuracy_times"] / s["accuracy_over"],
                                       rel=1e-14)
    assert r.full_index == 2 ** 64 - 1
    o.set_mixtures(False)
    r = o.search([g["mixtures_eq9_10"]["demand_mrps"]], s["slo_latency_us"], s["slo_accuracy"], 0)[0][0]
    assert r.cost == s["single_tuple_cost"] and r.choice2 == [0xFFFF, 0xFFFF] and r.replicas2 == [0, 0]


def small(seed, T=None):
    pb, se = workloads.tiny_mixture(seed, T)
    return pb, se, PyRef(pb)


@pytest.mark.parametrize("seed", range(24))
def test_objective_with_mixtures_matches_brute_force(seed):
    """Eq. 14 over options with their own accuracies (the paper's objective on the widened space)."""
    pb, se, ref = small(400 + seed)
    o = oracle.Oracle.from_problem(pb)
    o.set_mixtures(True)
    o.set_objective(1, 1.0, 0.035)
    cap = [4, 6, 9, 12][seed % 4] if pb.T == 3 else [6, 12, 24, 40][seed % 4]
    for D in se.demand_mrps.tolist():
        want, K, tr, margin = ref.search_mix(D, se.slo_latency_us, se.slo_accuracy, cap, objective=(1.0, 0.035))
        r = o.search([D], se.slo_latency_us, se.slo_accuracy, cap)[0][0]
        assert bool(r.feasible) == (want is not None)
        if want is None or (margin is not None and margin < 1e-9):
            continue
        if o.objective_margin(D, se.slo_latency_us, se.slo_accuracy, cap) < 1e-9:
            continue
        compare(r, want[:5], K, tr)
        assert r.objective == pytest.approx(float(want[5]), rel=1e-12, abs=1e-12)


def compare(r, want, K, truncated):
    ev = 1
    for k in K:
        ev *= k
    assert r.evaluated == ev and (r.flags & 1) == int(truncated)
    assert bool(r.feasible) == (want is not None)
    if want is None:
        return
    idx, cost, lat, acc, opts = want
    assert (r.index, r.cost, r.latency_us) == (idx, cost, lat)
    assert r.choice == [o["c1"] for o in opts] and r.choice2 == [o["c2"] for o in opts]
    assert r.replicas == [o["m1"] for o in opts] and r.replicas2 == [o["m2"] for o in opts]
    assert r.accuracy == pytest.approx(float(acc), rel=1e-12)


@pytest.mark.parametrize("seed", range(30))
def test_all_options_match_brute_force(seed):
    pb, se, ref = small(seed, T=1 + seed % 2)
    o = oracle.Oracle.from_problem(pb)
    o.set_mixtures(True)
    for D in se.demand_mrps.tolist()[:1 if pb.T == 2 else 2]:
        for t in range(pb.T):
            got, _ = o.options(D, se.slo_latency_us, 0, t)
            want = ref.mix_options(D, se.slo_latency_us, t)
            assert [(x[0], x[1], x[2], x[3], x[4], x[5]) for x in got] == \
                   [(w["c1"], w["c2"], w["m1"], w["m2"], w["lat"], w["cost"]) for w in want]
            assert [x[6] for x in got] == [w["acc"] for w in want]          # same fp64 formula, same bits
            for x, w in zip(got, want):
                assert x[6] == pytest.approx(float(w["accF"]), rel=1e-15)  # and the exact mean
        want, K, tr, margin = ref.search_mix(D, se.slo_latency_us, se.slo_accuracy, 0)
        if margin is not None and margin < 1e-9:
            continue
        compare(o.search([D], se.slo_latency_us, se.slo_accuracy, 0)[0][0], want, K, tr)


@pytest.mark.parametrize("seed", range(30))
def test_pruned_matches_second_implementation(seed):
    pb, se, ref = small(100 + seed)
    o = oracle.Oracle.from_problem(pb)
    o.set_mixtures(True)
    cap = [4, 6, 9, 12][seed % 4] if pb.T == 3 else [6, 12, 24, 40][seed % 4]
    for D in se.demand_mrps.tolist():
        lists, tr = ref.mix_lists(D, se.slo_latency_us, cap)
        for t in range(pb.T):
            got, gtr = o.options(D, se.slo_latency_us, cap, t)
            assert [(x[0], x[1], x[2], x[3]) for x in got] == [(w["c1"], w["c2"], w["m1"], w["m2"]) for w in lists[t]]
            assert len(got) <= cap
        want, K, tr, margin = ref.search_mix(D, se.slo_latency_us, se.slo_accuracy, cap)
        if margin is not None and margin < 1e-9:
            continue
        compare(o.search([D], se.slo_latency_us, se.slo_accuracy, cap)[0][0], want, K, tr)


@pytest.mark.parametrize("seed", range(20))
def test_invariants(seed):
    """Mixtures can only help: never costlier than single tuples; exact pruning keeps the
    optimal cost; a demand one replica carries leaves no mixture."""
    pb, se, ref = small(200 + seed, T=1 + seed % 2)
    pure = oracle.Oracle.from_problem(pb)
    mix = oracle.Oracle.from_problem(pb)
    mix.set_mixtures(True)
    for D in se.demand_mrps.tolist():
        a = pure.search([D], se.slo_latency_us, se.slo_accuracy, 0)[0][0]
        b = mix.search([D], se.slo_latency_us, se.slo_accuracy, 0)[0][0]
        if a.feasible:
            assert b.feasible and b.cost <= a.cost
        c = mix.search([D], se.slo_latency_us, se.slo_accuracy, 1 << 20)[0][0]     # prune, never thin
        assert c.flags == 0 and c.feasible == b.feasible and (not b.feasible or c.cost == b.cost)
        assert c.evaluated <= b.evaluated
    # demand below every tuple's throughput: the options are the single tuples
    low = int(pb.thr_mrps.min() * 1000 // int(pb.mult_milli.max()))
    if low >= 1:
        for t in range(pb.T):
            opts, _ = mix.options(low, se.slo_latency_us, 0, t)
            assert all(x[1] == 0xFFFF and x[2] == 1 for x in opts)
            assert len(opts) == sum(1 for p in range(pb.P) for _ in range(pb.V * pb.B)
                                    if pb.capacity_units == 0 or pb.units[p] <= pb.capacity_units)


def test_mixture_of_equal_variants_keeps_the_accuracy(g):
    """Two tuples of one variant: the weighted mean is that variant's accuracy (to rounding)."""
    o = make(g)
    opts, _ = o.options(260000, 100000, 0, 0)
    for x in opts:
        if x[1] != 0xFFFF and x[0] // 4 == x[1] // 4:
            assert x[6] == pytest.approx(g["accuracy"][0][x[0] // 4], rel=1e-15)


def test_capacity_drops_options_that_cannot_fit(g):
    o = make(g, capacity=4)
    opts, _ = o.options(260000, 100000, 0, 0)
    assert opts and all(x[5] <= 4 for x in opts)
    free, _ = make(g).options(260000, 100000, 0, 0)
    assert [x for x in free if x[5] <= 4] == opts


def test_argument_errors(g):
    o = make(g)
    with pytest.raises(oracle.OracleError):
        o.search([260000], 100000, 0.5, 1)                      # cap below 2
    o.set_factors(g["factors_eq4_5"]["factor_milli"])
    with pytest.raises(oracle.OracleError):
        o.search([260000], 100000, 0.5, 0)                      # not together with per-variant factors
    o.set_factors(None)
    o.set_search_space(True, True, False)
    with pytest.raises(oracle.OracleError):
        o.search([260000], 100000, 0.5, 0)                      # nor with static budgets
    o.set_search_space(True, True, True)
    o.set_mixtures(False)
    with pytest.raises(oracle.OracleError):
        o.options(260000, 100000, 0, 0)
