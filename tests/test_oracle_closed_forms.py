"""Pin 3: special cases with a closed form or a textbook algorithm, and the
prune against its second implementation on the full-size workloads."""
import numpy as np
import pytest

import oracle
from paper_2603_08797_amd import workloads as W
from pyref import PyRef

U32 = 2**32 - 1


def _chain(T, V, P, B, seed):
    r = W.SplitMix64(77, seed)
    lat = np.zeros((T, V, P, B), dtype=np.uint32)
    thr = np.zeros((T, V, P, B), dtype=np.uint32)
    for i in np.ndindex(T, V, P, B):
        lat[i] = r.randint(1, 30)          # small integers: the knapsack table stays tiny
        thr[i] = 1000 * r.randint(20, 300)
    acc = np.sort(0.6 + 0.4 * np.array([[r.uniform() for _ in range(V)] for _ in range(T)]), axis=1)
    units = np.arange(1, P + 1, dtype=np.uint32)
    batch = np.array([1 << b for b in range(B)], dtype=np.uint32)
    src = np.arange(0, T - 1, dtype=np.uint16)
    dst = np.arange(1, T, dtype=np.uint16)
    return W.Problem(T, V, P, B, units, batch, lat, thr, acc, src, dst,
                     np.full(T, 1000, dtype=np.uint32), 0, 2)


@pytest.mark.parametrize("seed", range(12))
def test_single_task_is_a_filtered_minimum(seed):
    pb = _chain(1, 3, 3, 2, seed)
    o = oracle.Oracle.from_problem(pb)
    D, slo_l, slo_a = 150_000, 30, 0.8
    rep, cost = o.cost_table(D)
    amax = pb.accuracy[0].max()
    ok = [(int(cost[0, c]), c) for c in range(pb.C)
          if 2 * int(pb.latency_us.reshape(1, -1)[0, c]) <= slo_l
          and pb.accuracy[0, c // (pb.P * pb.B)] / amax >= slo_a]
    res, bl, md = o.search([D], slo_l, slo_a, 0)
    if ok:
        assert (res[0].cost, res[0].index) == min(ok)
    else:
        assert not res[0].feasible


@pytest.mark.parametrize("seed", range(12))
def test_loose_slos_make_the_minimum_separable(seed):
    """No binding constraint: optimum cost = sum of per-task minima and the
    arg-min takes, per task, the lowest choice id among its minimisers."""
    pb, se = W.tiny_random(seed + 200, T=4)
    pb.capacity_units = 0
    o = oracle.Oracle.from_problem(pb)
    D = int(se.demand_mrps[-1])
    rep, cost = o.cost_table(D)
    res, _, _ = o.search([D], U32, 0.0, 0)
    r = res[0]
    assert r.feasible
    assert r.cost == int(cost.min(axis=1).sum())
    assert r.choice == [int(np.argmin(cost[t])) for t in range(pb.T)]


def test_unreachable_slos_are_infeasible_not_errors():
    pb, se = W.tiny_random(11, T=3)
    o = oracle.Oracle.from_problem(pb)
    D = int(se.demand_mrps[0])
    res, bl, md = o.search([D], U32, 1.0000001, 0)
    assert not res[0].feasible and bl == -1 and md == 0
    # latency SLO just below q * (critical path of the per-task minima)
    ref = PyRef(pb)
    fastest = [int(np.argmin(pb.latency_us.reshape(pb.T, -1)[t])) for t in range(pb.T)]
    floor = ref.latency(fastest)
    assert not o.search([D], floor - 1, 0.0, 0)[0][0].feasible
    pb.capacity_units = 0
    o2 = oracle.Oracle.from_problem(pb)
    r = o2.search([D], floor, 0.0, 0)[0][0]
    assert r.feasible and r.latency_us == floor


@pytest.mark.parametrize("seed", range(10))
def test_chain_without_accuracy_slo_is_a_multiple_choice_knapsack(seed):
    """Textbook DP over the latency budget gives the exact minimum cost."""
    T = 4
    pb = _chain(T, 2, 3, 2, seed)
    o = oracle.Oracle.from_problem(pb)
    D = 400_000
    rep, cost = o.cost_table(D)
    lat = pb.latency_us.reshape(T, -1)
    for slo_l in (40, 64, 90, 130, 240):
        budget = slo_l // 2
        INF = 10**9
        best = [0] + [INF] * budget           # best[w]: min cost with total latency exactly w
        for t in range(T):
            nxt = [INF] * (budget + 1)
            for w in range(budget + 1):
                if best[w] >= INF:
                    continue
                for c in range(pb.C):
                    w2 = w + int(lat[t, c])
                    if w2 <= budget:
                        nxt[w2] = min(nxt[w2], best[w] + int(cost[t, c]))
            best = nxt
        want = min(best)
        r = o.search([D], slo_l, 0.0, 0)[0][0]
        if want >= INF:
            assert not r.feasible
        else:
            assert r.feasible and r.cost == want


def test_diamond_with_equal_branches_reduces_to_a_chain_product():
    """All multipliers equal and the three branch tasks identical: every path
    has the same accuracy, so the system accuracy is one path's product."""
    w = W.diamond5()
    pb = w.problems[0]
    pb.mult_milli[:] = 1000
    pb.accuracy[2] = pb.accuracy[1]
    pb.accuracy[3] = pb.accuracy[1]
    o = oracle.Oracle.from_problem(pb)
    paths = o.paths()
    assert sorted(p for p, f in paths) == [[0, 1, 4], [0, 2, 4], [0, 3, 4]]
    assert all(f == pytest.approx(1 / 3, rel=1e-15) for p, f in paths)
    a = pb.accuracy
    amax = a[0, -1] * a[1, -1] * a[4, -1]
    for v0, vb, v4 in [(0, 0, 0), (1, 2, 3), (3, 1, 0)]:
        got = o.accuracy_of_variants([v0, vb, vb, vb, v4])
        assert got == pytest.approx(a[0, v0] * a[1, vb] * a[4, v4] / amax, rel=1e-14)


def test_diamond_request_fractions_follow_the_multipliers():
    o = oracle.Oracle.from_problem(W.diamond5().problems[0])
    got = {tuple(p): f for p, f in o.paths()}
    assert got == {(0, 1, 4): 0.5, (0, 2, 4): 0.25, (0, 3, 4): 0.25}


def test_request_fractions_sum_to_one_on_random_graphs():
    for seed in range(60):
        pb, _ = W.tiny_random(seed)
        o = oracle.Oracle.from_problem(pb)
        assert sum(f for _, f in o.paths()) == pytest.approx(1.0, rel=1e-14)
        assert o.accuracy_of_variants([int(np.argmax(pb.accuracy[t])) for t in range(pb.T)]) \
            == pytest.approx(1.0, rel=1e-15)


@pytest.mark.parametrize("name,levels,cap", [("diamond5", 32, None), ("diamond5", 16, 16),
                                             ("diamond5", 8, 9), ("xr8", 12, None),
                                             ("xr8", 6, 37), ("dagbatch", 10, None)])
def test_prune_lists_match_second_implementation(name, levels, cap):
    w = W.BENCH_WORKLOADS[name]()
    n_trunc = 0
    for pb, se in list(zip(w.problems, w.searches))[:levels if name == "dagbatch" else 1]:
        o = oracle.Oracle.from_problem(pb)
        ref = PyRef(pb)
        dem = se.demand_mrps.tolist()
        step = max(1, len(dem) // levels)
        pc = se.prune_cap if cap is None else cap
        for D in dem[::step]:
            lists, truncated = ref.lists(D, se.slo_latency_us, pc)
            n_trunc += truncated
            any_tr = False
            for t in range(pb.T):
                ids, tr = o.pruned(D, se.slo_latency_us, pc, t)
                any_tr |= tr
                assert ids.tolist() == lists[t]
                assert len(ids) <= pc
            assert any_tr == truncated
    if (name, cap) != ("diamond5", None):
        assert n_trunc > 0      # the cap does bind here


def test_thinning_keeps_fastest_and_cheapest_of_every_variant():
    w = W.xr8()
    pb, se = w.problems[0], w.searches[0]
    o = oracle.Oracle.from_problem(pb)
    lat = pb.latency_us.reshape(pb.T, -1)
    PB = pb.P * pb.B
    for D in se.demand_mrps[::9].tolist():
        rep, cost = o.cost_table(D)
        for t in range(pb.T):
            exact, _ = o.pruned(D, se.slo_latency_us, pb.C, t)      # cap = C: never thins
            thin, tr = o.pruned(D, se.slo_latency_us, se.prune_cap, t)
            assert set(thin.tolist()) <= set(exact.tolist())
            for v in range(pb.V):
                ev = [c for c in exact.tolist() if c // PB == v]
                tv = [c for c in thin.tolist() if c // PB == v]
                assert bool(ev) == bool(tv)
                if ev:
                    assert min(lat[t, c] for c in ev) == min(lat[t, c] for c in tv)
                    assert min(cost[t, c] for c in ev) == min(cost[t, c] for c in tv)
                    assert len(tv) <= max(se.prune_cap // pb.V, 0) or len(tv) == len(ev)
