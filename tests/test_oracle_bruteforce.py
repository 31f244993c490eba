"""Pin 2: the C oracle against an independent exact-arithmetic brute force
(tests/pyref.py) on many tiny random systems: diamonds, isolated tasks,
multi-source and multi-sink graphs, with and without pruning."""
import numpy as np
import pytest

import oracle
from paper_2603_08797_amd import workloads as W
from pyref import PyRef

SEEDS = list(range(160))


@pytest.mark.parametrize("seed", SEEDS)
def test_tiny_random(seed):
    pb, se = W.tiny_random(seed)
    o = oracle.Oracle.from_problem(pb)
    ref = PyRef(pb)
    assert o.amax() == pytest.approx(float(ref.amax), rel=1e-14)
    for D in se.demand_mrps.tolist():
        rep, cost = o.cost_table(D)
        for t in range(pb.T):
            for c in range(pb.C):
                assert (int(rep[t, c]), int(cost[t, c])) == ref.rep_cost(D, t, c)
        lists, truncated = ref.lists(D, se.slo_latency_us, se.prune_cap)
        for t in range(pb.T):
            ids, tr = o.pruned(D, se.slo_latency_us, se.prune_cap, t)
            assert ids.tolist() == lists[t]
        best, K, truncated, margin = ref.search(D, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
        if margin is not None and margin <= 1e-9:
            pytest.skip("accuracy within the guard band of the SLO")
        res, bl, md = o.search([D], se.slo_latency_us, se.slo_accuracy, se.prune_cap)
        r = res[0]
        Ko, space, tro = o.space(D, se.slo_latency_us, se.prune_cap)
        assert Ko.tolist() == K and tro == truncated
        assert r.evaluated == int(np.prod(np.array(K, dtype=object)))
        assert r.flags == int(truncated)
        if best is None:
            assert not r.feasible and bl == -1 and md == 0
        else:
            idx, cst, lat, acc, choice = best
            assert r.feasible and r.index == idx and r.cost == cst and r.latency_us == lat
            assert r.choice == choice
            assert r.accuracy == pytest.approx(float(acc), rel=1e-13)
            assert r.full_index == sum(c * pb.C ** t for t, c in enumerate(choice))
            assert r.replicas == [ref.rep_cost(D, t, choice[t])[0] for t in range(pb.T)]


@pytest.mark.parametrize("seed", SEEDS[:40])
def test_eval_every_candidate(seed):
    pb, se = W.tiny_random(seed)
    o = oracle.Oracle.from_problem(pb)
    ref = PyRef(pb)
    D = int(se.demand_mrps[0])
    lists, _ = ref.lists(D, se.slo_latency_us, se.prune_cap)
    K = [len(l) for l in lists]
    n = int(np.prod(K))
    if n == 0:
        pytest.skip("empty searched space")
    lat, rep, cost, acc, mask = o.eval(D, se.slo_latency_us, se.slo_accuracy, se.prune_cap,
                                       np.arange(n, dtype=np.uint64))
    from fractions import Fraction
    slo = Fraction(float(se.slo_accuracy))
    for i in range(n):
        j, choice = i, []
        for t in range(pb.T):
            choice.append(lists[t][j % K[t]])
            j //= K[t]
        assert lat[i] == ref.latency(choice)
        rc = [ref.rep_cost(D, t, choice[t]) for t in range(pb.T)]
        assert rep[i].tolist() == [x[0] for x in rc]
        assert cost[i] == sum(x[1] for x in rc)
        a = ref._acc([ref.variant(c) for c in choice]) / ref.amax
        assert acc[i] == pytest.approx(float(a), rel=1e-13)
        if abs(a - slo) > 1e-9:
            m = (1 if lat[i] <= se.slo_latency_us else 0) | (2 if a >= slo else 0)
            m |= 4 if (pb.capacity_units == 0 or cost[i] <= pb.capacity_units) else 0
            assert mask[i] == m


def test_search_range_is_the_restricted_argmin():
    pb, se = W.tiny_random(7, T=3)
    o = oracle.Oracle.from_problem(pb)
    D = int(se.demand_mrps[0])
    K, space, _ = o.space(D, se.slo_latency_us, 0)
    lat, rep, cost, acc, mask = o.eval(D, 10**9, 0.0, 0, np.arange(space, dtype=np.uint64))
    for lo, hi in [(0, space), (3, 11), (space // 2, space), (5, 6)]:
        r = o.search_range(D, 10**9, 0.0, 0, lo, hi, threads=3)
        ok = [(int(cost[i]), i) for i in range(lo, hi) if mask[i] == 7]
        if ok:
            assert (r.cost, r.index) == min(ok)
        else:
            assert not r.feasible


def test_threads_do_not_change_the_answer():
    w = W.chain3()
    pb, se = w.problems[0], w.searches[0]
    o = oracle.Oracle.from_problem(pb)
    a, _, _ = o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0, threads=1)
    b, _, _ = o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0, threads=5)
    assert a == b


def test_rejects_bad_input():
    pb, se = W.tiny_random(3, T=3)
    with pytest.raises(oracle.OracleError) as e:
        oracle.Oracle(3, pb.V, pb.P, pb.B, pb.units, pb.batch, pb.latency_us, pb.thr_mrps,
                      pb.accuracy, [0, 1, 2], [1, 2, 0], pb.mult_milli, 0, 2)
    assert e.value.code == oracle.E_CYCLE
    with pytest.raises(oracle.OracleError):
        oracle.Oracle(3, pb.V, pb.P, pb.B, pb.units, pb.batch, pb.latency_us, pb.thr_mrps,
                      pb.accuracy, [0, 0], [1, 1], pb.mult_milli, 0, 2)   # duplicate edge
    with pytest.raises(oracle.OracleError):
        oracle.Oracle(3, pb.V, pb.P, pb.B, pb.units, pb.batch, pb.latency_us, pb.thr_mrps,
                      pb.accuracy, [1], [1], pb.mult_milli, 0, 2)         # self loop
