"""Pins of the oracle's search-space restrictions (ablations A / S / T of Section 4.3,
static budgets of Appendix B)."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2603_08797_amd import workloads as W
from pyref import PyRef

COMBOS = list(itertools.product([True, False], repeat=3))
U32 = 2**32 - 1


def shares_clear(ref):
    sh = ref.resource_shares()
    if sh is None:
        return True
    return all(min(x - (x.numerator // x.denominator), 1 - (x - (x.numerator // x.denominator))) > 1e-9 for x in sh)


@pytest.mark.parametrize("seed", range(60))
def test_tiny_random_all_combinations(seed):
    pb, se = W.tiny_random(seed + 1300)
    if pb.capacity_units == 0 and seed % 2:
        pb.capacity_units = 6 * pb.T + seed % 7
    for A, S, T in COMBOS:
        o = oracle.Oracle.from_problem(pb)
        o.set_search_space(A, S, T)
        ref = PyRef(pb)
        ref.space = (A, S, T)
        if not shares_clear(ref):
            continue
        for D in se.demand_mrps.tolist():
            lists, truncated = ref.lists(D, se.slo_latency_us, se.prune_cap)
            for t in range(pb.T):
                ids, _ = o.pruned(D, se.slo_latency_us, se.prune_cap, t)
                assert ids.tolist() == lists[t], (A, S, T, t)
            best, K, _, margin = ref.search(D, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
            if margin is not None and margin <= 1e-9:
                continue
            r = o.search([D], se.slo_latency_us, se.slo_accuracy, se.prune_cap)[0][0]
            assert r.evaluated == int(np.prod(np.array(K, dtype=object)))
            if best is None:
                assert not r.feasible
            else:
                assert r.feasible and (r.index, r.cost, r.latency_us, r.choice) == (best[0], best[1], best[2], best[4])


def test_restrictions_only_shrink_the_space_and_raise_the_cost():
    w = W.chain3()
    pb, se = w.problems[0], w.searches[0]
    full = oracle.Oracle.from_problem(pb)
    base = full.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0, threads=4)[0][0]
    for A, S, T in COMBOS[1:]:
        o = oracle.Oracle.from_problem(pb)
        o.set_search_space(A, S, T)
        r = o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0, threads=4)[0][0]
        assert r.evaluated <= base.evaluated
        if r.feasible:
            assert base.feasible and r.cost >= base.cost
            # its winner is a candidate of the full space with the same scores
            lat, rep, cost, acc, mask = full.eval(int(se.demand_mrps[0]), se.slo_latency_us, se.slo_accuracy, 0,
                                                  [r.full_index])
            assert (lat[0], cost[0], mask[0]) == (r.latency_us, r.cost, 7)


def test_no_accuracy_scaling_pins_every_task_to_its_best_variant():
    w = W.diamond5()
    pb, se = w.problems[0], w.searches[0]
    o = oracle.Oracle.from_problem(pb)
    o.set_search_space(False, True, True)
    res = o.search(se.demand_mrps[:6], se.slo_latency_us, 0.0, 0, threads=8)[0]
    for r in res:
        assert r.feasible and r.accuracy == pytest.approx(1.0, rel=1e-15)
        assert all(c // (pb.P * pb.B) == pb.V - 1 for c in r.choice)     # accuracies ascend with v
    K, space, _ = o.space(int(se.demand_mrps[0]), se.slo_latency_us, 0)
    assert K.tolist() == [pb.P * pb.B] * pb.T


def test_no_partitioning_uses_whole_gpus_only():
    w = W.chain4()
    pb, se = w.problems[0], w.searches[0]
    o = oracle.Oracle.from_problem(pb)
    o.set_search_space(True, False, True)
    K, space, _ = o.space(int(se.demand_mrps[0]), se.slo_latency_us, 0)
    assert K.tolist() == [pb.V * pb.B] * pb.T
    ids, _ = o.pruned(int(se.demand_mrps[0]), se.slo_latency_us, 0, 2)
    assert all((c // pb.B) % pb.P == pb.P - 1 for c in ids.tolist())      # 7 of 7 units


def test_static_budgets_imply_the_global_constraints():
    """With per-task budgets every combination of surviving choices meets Eq. 3 and Eq. 8."""
    for seed in range(25):
        pb, se = W.tiny_random(seed + 1400, T=3)
        pb.capacity_units = 20 + seed
        o = oracle.Oracle.from_problem(pb)
        o.set_search_space(True, True, False)
        if o.budget_margin() <= 1e-9:
            continue
        for D in se.demand_mrps.tolist():
            K, space, _ = o.space(D, se.slo_latency_us, 0)
            if space == 0:
                continue
            lat, rep, cost, acc, mask = o.eval(D, se.slo_latency_us, 0.0, 0, np.arange(space, dtype=np.uint64))
            assert np.all(mask & 1) and np.all(mask & 4)


def test_a_single_task_keeps_the_whole_budget():
    pb, se = W.tiny_random(3, T=1)
    pb.capacity_units = 9
    a, b = oracle.Oracle.from_problem(pb), oracle.Oracle.from_problem(pb)
    b.set_search_space(True, True, False)
    for D in se.demand_mrps.tolist():
        ra = a.search([D], se.slo_latency_us, se.slo_accuracy, 0)[0][0]
        rb = b.search([D], se.slo_latency_us, se.slo_accuracy, 0)[0][0]
        assert (ra.feasible, ra.cost, ra.choice) == (rb.feasible, rb.cost, rb.choice)
