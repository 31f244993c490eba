"""GPU parity of the search-space restrictions (ablations A / S / T) against the oracle."""
import itertools

import numpy as np
import pytest

import oracle
from paper_2603_08797_amd import jsv, workloads as W
from test_gpu_parity import same

pytestmark = pytest.mark.gpu
COMBOS = list(itertools.product([True, False], repeat=3))
THREADS = 16


@pytest.fixture(scope="module")
def ctx():
    j = jsv.Jsv(device=0)
    yield j
    j.set_search_space(True, True, True)
    j.close()


def run(j, pb, se, space, threads=THREADS, dem=None):
    dem = se.demand_mrps if dem is None else dem
    o = oracle.Oracle.from_problem(pb)
    o.set_search_space(*space)
    if o.budget_margin() <= 1e-9:
        return None
    j.set_search_space(*space)
    j.load(pb)
    res, summ = j.search(dem, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    ref, bl, md = o.search(dem, se.slo_latency_us, se.slo_accuracy, se.prune_cap, threads=threads)
    for l, (a, b) in enumerate(zip(res, ref)):
        same(a, b, f"{space} level {l}")
    assert (summ.best_level, summ.max_demand_mrps) == (bl, md)
    for t in range(pb.T):
        a, _ = j.get_pruned(int(dem[0]), se.slo_latency_us, se.prune_cap, t)
        b, _ = o.pruned(int(dem[0]), se.slo_latency_us, se.prune_cap, t)
        assert a.tolist() == b.tolist()
    return res, summ


@pytest.mark.parametrize("seed", range(40))
def test_tiny_random_all_combinations(ctx, seed):
    pb, se = W.tiny_random(seed + 1300)
    if pb.capacity_units == 0 and seed % 2:
        pb.capacity_units = 6 * pb.T + seed % 7
    if oracle.Oracle.from_problem(pb).accuracy_margin(se.slo_accuracy) <= 1e-9:
        pytest.skip("inside the accuracy guard band")
    for space in COMBOS:
        run(ctx, pb, se, space, threads=1)


@pytest.mark.parametrize("space", COMBOS)
def test_chain3_and_diamond5(ctx, space):
    w = W.chain3()
    run(ctx, w.problems[0], w.searches[0], space)
    w = W.diamond5()
    run(ctx, w.problems[0], w.searches[0], space)


def test_flags_persist_across_loads_and_reset(ctx):
    w = W.chain3()
    pb, se = w.problems[0], w.searches[0]
    full, _ = run(ctx, pb, se, (True, True, True))
    ctx.set_search_space(False, False, True)
    ctx.load(pb)                                   # a new load keeps the restriction
    r, _ = ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0)
    assert r[0].evaluated == pb.B ** 3 and r[0].evaluated < full[0].evaluated
    ctx.set_search_space(True, True, True)         # switching back needs no reload
    r, _ = ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0)
    assert r[0] == full[0]


def test_batch_with_restrictions(ctx):
    w = W.dagbatch(n=40)
    for pb, se in zip(w.problems, w.searches):
        se.prune_cap = 12
    for space in [(False, True, True), (True, False, False)]:
        ctx.set_search_space(*space)
        res = ctx.search_batch(w.problems, w.searches)
        for k, (pb, se, a) in enumerate(zip(w.problems, w.searches, res)):
            o = oracle.Oracle.from_problem(pb)
            o.set_search_space(*space)
            if o.budget_margin() <= 1e-9:
                continue
            b = o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap, threads=THREADS)[0][0]
            same(a, b, f"{space} problem {k}")
    ctx.set_search_space(True, True, True)


def test_max_serviceable_demand_by_search_space(ctx):
    """The analysis of Fig. 3 on a synthetic traffic-analysis-like graph (detector feeding
    two classifiers, one of them run twice per detection) on a large testbed: the full space
    serves at least as much demand as any restricted one, and every GPU value is the oracle's."""
    w = W.diamond5()
    pb = w.problems[0]
    T = 3
    small = W.Problem(T, pb.V, pb.P, pb.B, pb.units, pb.batch, pb.latency_us[:T].copy(), pb.thr_mrps[:T].copy(),
                      pb.accuracy[:T].copy(), np.array([0, 0], dtype=np.uint16), np.array([1, 2], dtype=np.uint16),
                      np.array([1000, 2000, 1000], dtype=np.uint32), 840, 2)
    dem = np.array([int(round(1000 * 5.0 * 1.25 ** i)) for i in range(40)], dtype=np.uint32)
    se = W.Search(dem, 120_000, 0.9, 0)
    if oracle.Oracle.from_problem(small).accuracy_margin(0.9) <= 1e-9:
        pytest.skip("inside the accuracy guard band")
    best = {}
    for space in COMBOS:
        out = run(ctx, small, se, space)
        if out is not None:
            best[space] = out[1].max_demand_mrps
    full = best[(True, True, True)]
    assert full > 0 and all(v <= full for v in best.values())
    assert best[(False, False, False)] == min(best.values())
