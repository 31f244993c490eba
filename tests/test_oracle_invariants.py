"""Pin 4: properties that follow from the formulation (Section 3.2): latency
and accuracy do not depend on demand, cost is a sum of per-task terms that
grow with demand, and constraints are inclusive."""
import numpy as np
import pytest

import oracle
from paper_2603_08797_amd import workloads as W

U32 = 2**32 - 1


def _cost(r):
    return r.cost if r.feasible else None


@pytest.mark.parametrize("seed", range(30))
def test_cost_is_monotone_in_both_slos_and_in_demand(seed):
    pb, se = W.tiny_random(seed + 400, T=3)
    o = oracle.Oracle.from_problem(pb)
    D = int(se.demand_mrps[0])
    prev = None
    for slo_l in range(4000, 90000, 6000):          # loosening latency
        c = _cost(o.search([D], slo_l, se.slo_accuracy, 0)[0][0])
        if prev is not None:
            assert c is not None and c <= prev
        prev = c if c is not None else prev
    prev = None
    for slo_a in (0.99, 0.9, 0.8, 0.7, 0.5, 0.2, 0.0):   # loosening accuracy
        c = _cost(o.search([D], se.slo_latency_us, slo_a + 1e-7, 0)[0][0])
        if prev is not None:
            assert c is not None and c <= prev
        prev = c if c is not None else prev
    levels = [1000 * k for k in (1, 5, 20, 60, 150, 400, 900)]
    res, bl, md = o.search(levels, se.slo_latency_us, se.slo_accuracy, 0)
    costs = [_cost(r) for r in res]
    feas = [c is not None for c in costs]
    assert feas == sorted(feas, reverse=True)        # feasible levels form a prefix
    got = [c for c in costs if c is not None]
    assert got == sorted(got)
    if any(feas):
        assert bl == feas.count(True) - 1 and md == levels[bl]


@pytest.mark.parametrize("seed", range(10))
def test_latency_and_accuracy_bits_do_not_depend_on_demand(seed):
    pb, se = W.tiny_random(seed + 500, T=3)
    o = oracle.Oracle.from_problem(pb)
    K, space, _ = o.space(1000, U32, 0)
    idx = np.arange(space, dtype=np.uint64)
    a = o.eval(1000, se.slo_latency_us, se.slo_accuracy, 0, idx)
    b = o.eval(777000, se.slo_latency_us, se.slo_accuracy, 0, idx)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[3], b[3])
    assert np.array_equal(a[4] & 3, b[4] & 3)
    assert np.all(b[2] >= a[2])                      # cost grows with demand
    assert np.all((b[4] & 4) <= (a[4] & 4))          # feasible at D => feasible below D


@pytest.mark.parametrize("seed", range(40))
def test_pruned_optimum_equals_exhaustive_optimum_unless_thinned(seed):
    pb, se = W.tiny_random(seed + 600)
    o = oracle.Oracle.from_problem(pb)
    cap = max(2 * pb.V, pb.C // 2)
    for D in se.demand_mrps.tolist():
        full = o.search([D], se.slo_latency_us, se.slo_accuracy, 0)[0][0]
        pr = o.search([D], se.slo_latency_us, se.slo_accuracy, cap)[0][0]
        if pr.flags & 1:
            assert (not pr.feasible) or (full.feasible and pr.cost >= full.cost)
        else:
            assert pr.feasible == full.feasible
            assert _cost(pr) == _cost(full)
        if pr.feasible:                              # the winner is a real candidate
            assert pr.full_index == sum(c * pb.C ** t for t, c in enumerate(pr.choice))
            lat, rep, cost, acc, mask = o.eval(D, se.slo_latency_us, se.slo_accuracy, 0,
                                               [pr.full_index])
            assert mask[0] == 7 and cost[0] == pr.cost and lat[0] == pr.latency_us


def test_scaling_demand_and_throughput_together_changes_nothing():
    pb, se = W.tiny_random(42, T=3)
    pb.thr_mrps = (pb.thr_mrps // 8).astype(np.uint32)
    o1 = oracle.Oracle.from_problem(pb)
    pb2, _ = W.tiny_random(42, T=3)
    pb2.thr_mrps = ((pb2.thr_mrps // 8) * 5).astype(np.uint32)
    o2 = oracle.Oracle.from_problem(pb2)
    for D in (3000, 41000, 250000):
        a = o1.search([D], se.slo_latency_us, se.slo_accuracy, 0)[0][0]
        b = o2.search([5 * D], se.slo_latency_us, se.slo_accuracy, 0)[0][0]
        assert a == b


@pytest.mark.parametrize("seed", range(12))
def test_relabelling_tasks_keeps_cost_latency_accuracy(seed):
    pb, se = W.tiny_random(seed + 700, T=4)
    perm = [2, 0, 3, 1]                      # new id of old task t
    inv = [perm.index(i) for i in range(4)]  # old id of new task i
    o1 = oracle.Oracle.from_problem(pb)
    o2 = oracle.Oracle(pb.T, pb.V, pb.P, pb.B, pb.units, pb.batch, pb.latency_us[inv],
                       pb.thr_mrps[inv], pb.accuracy[inv],
                       [perm[a] for a in pb.src.tolist()], [perm[b] for b in pb.dst.tolist()],
                       pb.mult_milli[inv], pb.capacity_units, pb.queue_factor)
    assert o1.amax() == pytest.approx(o2.amax(), rel=1e-14)
    for D in se.demand_mrps.tolist():
        a = o1.search([D], se.slo_latency_us, se.slo_accuracy, 0)[0][0]
        b = o2.search([D], se.slo_latency_us, se.slo_accuracy, 0)[0][0]
        assert a.feasible == b.feasible
        if a.feasible:
            assert a.cost == b.cost
            # the winners may differ among equal-cost candidates; score a's winner under b's labels
            idx = sum(a.choice[inv[i]] * pb.C ** i for i in range(4))
            lat, rep, cost, acc, mask = o2.eval(D, se.slo_latency_us, se.slo_accuracy, 0, [idx])
            assert lat[0] == a.latency_us and cost[0] == a.cost and mask[0] == 7
            assert acc[0] == pytest.approx(a.accuracy, rel=1e-13)


def test_bounds_are_inclusive():
    pb, se = W.tiny_random(5, T=2)
    pb.capacity_units = 0
    o = oracle.Oracle.from_problem(pb)
    D = int(se.demand_mrps[0])
    r = o.search([D], U32, 0.0, 0)[0][0]
    # tighten each bound to exactly the winner's value: it must stay feasible
    assert o.search([D], r.latency_us, 0.0, 0)[0][0].feasible
    pb.capacity_units = r.cost
    o2 = oracle.Oracle.from_problem(pb)
    r2 = o2.search([D], U32, 0.0, 0)[0][0]
    assert r2.feasible and r2.cost == r.cost
    pb.capacity_units = r.cost - 1
    assert not oracle.Oracle.from_problem(pb).search([D], U32, 0.0, 0)[0][0].feasible
    # accuracy: the all-best-variants candidate has A_obj = A_max/A_max = 1.0 exactly
    assert o.search([D], U32, 1.0, 0)[0][0].feasible
