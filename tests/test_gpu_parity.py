"""GPU parity: the HIP library (through its C ABI) against the CPU oracle.

Integers (latency, replicas, cost, mask, arg-min index, choices) must be
bit-exact; fp64 accuracy within 1e-12 relative.
"""
import numpy as np
import pytest

import oracle
from paper_2603_08797_amd import jsv, workloads as W

pytestmark = pytest.mark.gpu
REL = 1e-12


@pytest.fixture(scope="module")
def ctx():
    j = jsv.Jsv(device=0)
    yield j
    j.close()


def same(a, b, where=""):
    assert a.feasible == b.feasible, where
    assert a.evaluated == b.evaluated, where
    assert a.flags & 1 == b.flags, where          # bit1 only tells which key width ran
    assert a.index == b.index, (where, a, b)
    assert a.full_index == b.full_index, where
    assert a.cost == b.cost and a.latency_us == b.latency_us, where
    assert a.choice == b.choice and a.replicas == b.replicas, where
    assert abs(a.accuracy - b.accuracy) <= REL * abs(b.accuracy), where


def check_search(j, pb, se, threads=16):
    j.load(pb)
    res, summ = j.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    o = oracle.Oracle.from_problem(pb)
    ref, bl, md = o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap, threads=threads)
    for l, (a, b) in enumerate(zip(res, ref)):
        same(a, b, f"level {l}")
    assert (summ.best_level, summ.max_demand_mrps) == (bl, md)
    return res, summ


def test_hand_worked_chain(ctx):
    import json, os
    with open(os.path.join(os.path.dirname(__file__), "golden", "p1_two_task_chain.json")) as f:
        g = json.load(f)
    lat = np.array(g["latency_us"], dtype=np.uint32)
    acc = np.array(g["accuracy"])
    ctx.load_profile(2, 2, 2, 2, g["units"], g["batch"], lat, None, acc)
    ctx.set_dag(2, [0], [1], g["mult_milli"], 0, 2)
    for s in g["at_260_rps"]["searches"]:
        res, summ = ctx.search([g["at_260_rps"]["demand_mrps"]], s["slo_latency_us"], s["slo_accuracy"], 0)
        r = res[0]
        assert (r.index, r.choice, r.cost, r.latency_us) == (s["index"], s["choice"], s["cost"], s["latency_us"])
        assert abs(r.accuracy - s["accuracy_num"] / s["accuracy_den"]) < 1e-14
    sw = g["sweep"]
    ctx.set_dag(2, [0], [1], g["mult_milli"], sw["capacity_units"], 2)
    res, summ = ctx.search(sw["demand_mrps"], sw["slo_latency_us"], sw["slo_accuracy"], 0)
    assert [r.index if r.feasible else None for r in res] == sw["index"]
    assert [r.cost if r.feasible else None for r in res] == sw["cost"]
    assert (summ.best_level, summ.max_demand_mrps) == (sw["best_level"], sw["max_demand_mrps"])


@pytest.mark.parametrize("seed", range(120))
def test_tiny_random(ctx, seed):
    pb, se = W.tiny_random(seed)
    o = oracle.Oracle.from_problem(pb)
    if o.accuracy_margin(se.slo_accuracy) <= 1e-9:
        pytest.skip("inside the accuracy guard band")
    check_search(ctx, pb, se, threads=1)
    for D in se.demand_mrps.tolist():
        for t in range(pb.T):
            a, ta = ctx.get_pruned(D, se.slo_latency_us, se.prune_cap, t)
            b, tb = o.pruned(D, se.slo_latency_us, se.prune_cap, t)
            assert a.tolist() == b.tolist() and ta == tb
        K, space, _ = o.space(D, se.slo_latency_us, se.prune_cap)
        if space:
            idx = np.arange(min(space, 4096), dtype=np.uint64)
            ga = ctx.eval_candidates(D, se.slo_latency_us, se.slo_accuracy, se.prune_cap, idx)
            gb = o.eval(D, se.slo_latency_us, se.slo_accuracy, se.prune_cap, idx)
            for x, y in zip((ga[0], ga[1], ga[2], ga[4]), (gb[0], gb[1], gb[2], gb[4])):
                assert np.array_equal(x, y)
            assert np.all(np.abs(ga[3] - gb[3]) <= REL * np.abs(gb[3]))


def test_chain3_exhaustive(ctx):
    w = W.chain3()
    check_search(ctx, w.problems[0], w.searches[0])


def test_chain3_every_candidate(ctx):
    w = W.chain3()
    pb, se = w.problems[0], w.searches[0]
    ctx.load(pb)
    o = oracle.Oracle.from_problem(pb)
    D = int(se.demand_mrps[0])
    idx = np.arange(pb.C ** 3, dtype=np.uint64)
    ga = ctx.eval_candidates(D, se.slo_latency_us, se.slo_accuracy, 0, idx)
    gb = o.eval(D, se.slo_latency_us, se.slo_accuracy, 0, idx)
    for x, y in zip((ga[0], ga[1], ga[2], ga[4]), (gb[0], gb[1], gb[2], gb[4])):
        assert np.array_equal(x, y)
    assert np.all(np.abs(ga[3] - gb[3]) <= REL * np.abs(gb[3]))


def test_diamond5_sweep(ctx):
    w = W.diamond5()
    res, summ = check_search(ctx, w.problems[0], w.searches[0])
    assert any(r.feasible for r in res) and not all(r.feasible for r in res)


def test_chain4_exhaustive(ctx):
    w = W.chain4()
    res, summ = check_search(ctx, w.problems[0], w.searches[0])
    assert res[0].evaluated == 140 ** 4


def test_records_as_the_library_wrote_them(ctx):
    """raw=True hands back the C records without turning them into Python objects (what bench.py
    times); results() of them is what the plain call returns, for one system and for a batch."""
    w = W.diamond5(seed=0)
    pb, se = w.problems[0], w.searches[0]
    ctx.load(pb)
    want, wsum = ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    rec, rsum = ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap, raw=True)
    assert rec.shape == (len(se.demand_mrps),) and ctx.results(rec) == want
    assert (rsum.best_level, rsum.max_demand_mrps) == (wsum.best_level, wsum.max_demand_mrps)
    assert [int(c) for c in rec["cost_units"]] == [r.cost if r.feasible else 2**31 - 1 for r in want]
    b = W.dagbatch(seed=0)
    j = jsv.Jsv(device=0)
    try:
        j.load_batch(b.problems[:24], b.searches[:24])
        got, _ = j.search_loaded_batch()
        rec, _ = j.search_loaded_batch(raw=True)
        assert j.results(rec, batch=True) == got
    finally:
        j.close()
