"""GPU parity of the per-variant multiplicative factors (Eq. 4, 5) against the oracle."""
import json
import os

import numpy as np
import pytest

import oracle
from paper_2603_08797_amd import jsv, workloads
from test_gpu_parity import same

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def ctx():
    j = jsv.Jsv(device=0)
    yield j
    j.close()


def check(ctx, pb, se, fac, cap, objective=None, levels=None):
    D = se.demand_mrps if levels is None else se.demand_mrps[:levels]
    o = oracle.Oracle.from_problem(pb)
    o.set_factors(fac)
    ctx.load(pb)
    ctx.set_factors(fac)
    if objective:
        o.set_objective(1, *objective)
        ctx.set_objective(1, *objective)
    try:
        want, wbl, wmd = o.search(D, se.slo_latency_us, se.slo_accuracy, cap, threads=16)
        got, summ = ctx.search(D, se.slo_latency_us, se.slo_accuracy, cap)
    finally:
        ctx.set_objective(0, 1.0, 0.035)
    skipped = 0
    for l, (w, g) in enumerate(zip(want, got)):
        if objective and w.feasible and \
                o.objective_margin(int(D[l]), se.slo_latency_us, se.slo_accuracy, cap) < 1e-9:
            skipped += 1
            continue
        same(g, w, f"level {l}")
        assert g.index == g.full_index or not g.feasible
    if not skipped:
        assert (summ.best_level, summ.max_demand_mrps) == (wbl, wmd)
    return want


def test_hand_worked_chain(ctx):
    with open(os.path.join(HERE, "golden", "p1_two_task_chain.json")) as f:
        g = json.load(f)
    lat = np.array(g["latency_us"], dtype=np.uint32).reshape(g["T"], g["V"], g["P"], g["B"])
    ctx.load_profile(g["T"], g["V"], g["P"], g["B"], g["units"], g["batch"], lat, None,
                     np.array(g["accuracy"], dtype=np.float64))
    ctx.set_dag(g["T"], [0], [1], g["mult_milli"], 0, g["queue_factor"])
    f = g["factors_eq4_5"]
    ctx.set_factors(f["factor_milli"])
    for s in f["searches"]:
        res, summ = ctx.search([f["demand_mrps"]], s["slo_latency_us"], s["slo_accuracy"], 0)
        r = res[0]
        assert r.feasible and r.evaluated == 64
        assert (r.index, r.full_index, r.choice[:2], r.cost, r.latency_us, r.replicas[:2]) == \
               (s["index"], s["index"], s["choice"], s["cost"], s["latency_us"], s["replicas"])
    ob = f["objective"]
    ctx.set_objective(1, ob["alpha"], ob["beta"])
    try:
        r = ctx.search([f["demand_mrps"]], ob["slo_latency_us"], ob["slo_accuracy"], 0)[0][0]
    finally:
        ctx.set_objective(0, 1.0, 0.035)
    assert (r.index, r.choice[:2], r.cost) == (ob["index"], ob["choice"], ob["cost"])
    # back to fixed multipliers
    ctx.set_factors(None)
    s = f["searches"][1]
    r = ctx.search([f["demand_mrps"]], s["slo_latency_us"], s["slo_accuracy"], 0)[0][0]
    assert (r.index, r.cost) == (s["fixed_factor_answer"]["index"], s["fixed_factor_answer"]["cost"])


@pytest.mark.parametrize("seed", range(60))
def test_tiny_random(ctx, seed):
    k = 0
    while True:
        pb, se = workloads.tiny_random(7000 + 100 * seed + k)
        if pb.E > 0:
            break
        k += 1
    tails = sorted(set(int(a) for a in pb.src))
    varying = None if seed % 3 else tails[:1]
    fac = workloads.random_factors(pb, seed, varying=varying)
    check(ctx, pb, se, fac, se.prune_cap if seed % 2 else 0,
          objective=(1.0, 0.035) if seed % 5 == 4 else None)


@pytest.mark.parametrize("seed", range(3))
def test_diamond_pruned(ctx, seed):
    """5-task diamond: the source and one branch change downstream demands (16 combinations)."""
    w = workloads.diamond5(seed=seed, prune_cap=8)
    pb, se = w.problems[0], w.searches[0]
    fac = workloads.random_factors(pb, seed, varying=[0, 2])
    want = check(ctx, pb, se, fac, 8, levels=6)
    assert any(r.feasible for r in want)


def test_traffic3_exhaustive_levels(ctx):
    """Detector -> two classifiers at full size: 245^3 candidates per level, 5 combinations."""
    w = workloads.traffic3(seed=0, n_levels=4)
    pb, se, fac = w.problems[0], w.searches[0], w.meta["factor_milli"]
    want = check(ctx, pb, se, fac, 0)
    assert all(r.evaluated == 245 ** 3 for r in want)
    assert any(r.feasible for r in want)


def test_state_and_argument_errors(ctx):
    pb, se = workloads.tiny_random(7000)
    while pb.E == 0:
        pb, se = workloads.tiny_random(7001 + pb.T)
    ctx.load(pb)
    fac = workloads.random_factors(pb, 0)
    bad = fac.copy(); bad[0, 0] = 0
    with pytest.raises(jsv.JsvError):
        ctx.set_factors(bad)
    bad[0, 0] = 1_000_001
    with pytest.raises(jsv.JsvError):
        ctx.set_factors(bad)
    with pytest.raises(ValueError):
        ctx.set_factors(fac[:, :0])
    ctx.set_factors(fac)
    with pytest.raises(jsv.JsvError):
        ctx.get_pruned(int(se.demand_mrps[0]), se.slo_latency_us, 0, 0)
    ctx.set_search_space(True, True, False)
    try:
        with pytest.raises(jsv.JsvError):
            ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0)
    finally:
        ctx.set_search_space(True, True, True)
    # a new graph drops the factors
    ctx.set_dag(pb.T, pb.src, pb.dst, pb.mult_milli, pb.capacity_units, pb.queue_factor)
    o = oracle.Oracle.from_problem(pb)
    want = o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0)[0]
    got = ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0)[0]
    for w_, g_ in zip(want, got):
        same(g_, w_)


def test_demand_beyond_the_flow_range_is_an_overflow_on_both_sides(ctx):
    with open(os.path.join(HERE, "golden", "p1_two_task_chain.json")) as f:
        g = json.load(f)
    lat = np.array(g["latency_us"], dtype=np.uint32).reshape(g["T"], g["V"], g["P"], g["B"])
    acc = np.array(g["accuracy"], dtype=np.float64)
    o = oracle.Oracle(g["T"], g["V"], g["P"], g["B"], g["units"], g["batch"], lat, None, acc, [0], [1],
                      g["mult_milli"], 0, g["queue_factor"])
    o.set_factors([[1_000_000, 1_000_000]])
    with pytest.raises(oracle.OracleError) as e:
        o.search([4_000_000_000], 100000, 0.0, 0)
    assert e.value.code == -3
    ctx.load_profile(g["T"], g["V"], g["P"], g["B"], g["units"], g["batch"], lat, None, acc)
    ctx.set_dag(g["T"], [0], [1], g["mult_milli"], 0, g["queue_factor"])
    ctx.set_factors([[1_000_000, 1_000_000]])
    with pytest.raises(jsv.JsvError) as e:
        ctx.search([4_000_000_000], 100000, 0.0, 0)
    assert e.value.code == jsv.E_OVERFLOW
    # a demand just inside the range is searched on both sides
    want = o.search([17_000], 100000, 0.0, 0)[0][0]
    got = ctx.search([17_000], 100000, 0.0, 0)[0][0]
    same(got, want)
