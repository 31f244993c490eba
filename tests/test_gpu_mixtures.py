"""GPU parity of the two-tuple mixtures (Eq. 2, 6, 7, 9, 10) against the oracle."""
import dataclasses
import json
import os
import time

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
    j.set_mixtures(True)
    yield j
    j.close()


def check(ctx, pb, se, cap, levels=None, threads=16, margin=True, objective=None):
    D = se.demand_mrps if levels is None else se.demand_mrps[:levels]
    o = oracle.Oracle.from_problem(pb)
    o.set_mixtures(True)
    ctx.load(pb)
    if objective:
        o.set_objective(1, *objective)
        ctx.set_objective(1, *objective)
    try:
        want, wbl, wmd = o.search(D, se.slo_latency_us, se.slo_accuracy, cap, threads=threads)
        got, summ = ctx.search(D, se.slo_latency_us, se.slo_accuracy, cap)
    finally:
        ctx.set_objective(0, 1.0, 0.035)
    skipped = 0
    for l, (w, g) in enumerate(zip(want, got)):
        if margin and o.mixture_margin(int(D[l]), se.slo_latency_us, se.slo_accuracy, cap) < 1e-9:
            skipped += 1
            continue
        if objective and w.feasible and o.objective_margin(int(D[l]), se.slo_latency_us, se.slo_accuracy, cap) < 1e-9:
            skipped += 1
            continue
        same(g, w, f"level {l}")
        assert (g.choice2, g.replicas2) == (w.choice2, w.replicas2), f"level {l}"
        assert g.full_index == 2 ** 64 - 1
    if not skipped:
        assert (summ.best_level, summ.max_demand_mrps) == (wbl, wmd)
    return want


def test_hand_worked_chain(ctx):
    with open(os.path.join(HERE, "golden", "p1_two_task_chain.json")) as f:
        g = json.load(f)
    lat = np.array(g["latency_us"], dtype=np.uint32).reshape(g["T"], g["V"], g["P"], g["B"])
    acc = np.array(g["accuracy"], dtype=np.float64)
    s = g["mixtures_eq9_10"]["search"]
    D = g["mixtures_eq9_10"]["demand_mrps"]
    ctx.load_profile(g["T"], g["V"], g["P"], g["B"], g["units"], g["batch"], lat, None, acc)
    ctx.set_dag(g["T"], [0], [1], g["mult_milli"], 12, g["queue_factor"])
    r = ctx.search([D], s["slo_latency_us"], s["slo_accuracy"], 64)[0][0]
    assert r.feasible and r.cost == s["cost"] and not (r.flags & 1)
    o = oracle.Oracle(g["T"], g["V"], g["P"], g["B"], g["units"], g["batch"], lat, None, acc, [0], [1],
                      g["mult_milli"], 12, g["queue_factor"])
    o.set_mixtures(True)
    w = o.search([D], s["slo_latency_us"], s["slo_accuracy"], 64)[0][0]
    same(r, w)
    assert (r.choice2, r.replicas2) == (w.choice2, w.replicas2)


@pytest.mark.parametrize("seed", range(80))
def test_tiny_mixture(ctx, seed):
    pb, se = workloads.tiny_mixture(3000 + seed)
    if pb.capacity_units == 0:
        pb = dataclasses.replace(pb, capacity_units=30)
    cap = [2, 4, 7, 12, 40, 400][seed % 6]
    check(ctx, pb, se, cap)


@pytest.mark.parametrize("seed", range(40))
def test_objective_over_mixtures(ctx, seed):
    pb, se = workloads.tiny_mixture(3500 + seed)
    if pb.capacity_units == 0:
        pb = dataclasses.replace(pb, capacity_units=30)
    check(ctx, pb, se, [4, 7, 12, 40][seed % 4], objective=(1.0, 0.035))


def first(name, seed=0):
    w = workloads.BENCH_WORKLOADS[name](seed=seed)
    return w.problems[0], w.searches[0]


@pytest.mark.parametrize("cap", [12, 16])
def test_chain3_sized(ctx, cap):
    """48 tuples per task: up to 5600 options per task, thinned to cap; mixtures win."""
    pb, se = first("chain3")
    se = dataclasses.replace(se, demand_mrps=np.array([100_000, 200_000, 300_000], dtype=np.uint32), slo_accuracy=0.9)
    want = check(ctx, pb, se, cap)
    assert any(r.feasible for r in want) and any(r.flags & 1 for r in want)
    assert any(c != 0xFFFF for r in want if r.feasible for c in r.choice2)


def test_diamond5_sized(ctx):
    """140 tuples per task, 5 tasks, 56 units."""
    pb, se = first("diamond5")
    se = dataclasses.replace(se, demand_mrps=se.demand_mrps[[12, 20, 24]], slo_accuracy=0.9)
    t0 = time.time()
    want = check(ctx, pb, se, 16)
    print(f"diamond5 mixtures: {time.time() - t0:.1f} s", flush=True)
    assert any(r.feasible for r in want)


def test_argument_and_state_errors(ctx):
    pb, se = workloads.tiny_mixture(3000)
    pb = dataclasses.replace(pb, capacity_units=30)
    ctx.load(pb)
    D = se.demand_mrps
    for cap in (0, 1, 4096):
        with pytest.raises(jsv.JsvError):
            ctx.search(D, se.slo_latency_us, se.slo_accuracy, cap)
    with pytest.raises(jsv.JsvError):
        ctx.get_pruned(int(D[0]), se.slo_latency_us, 8, 0)
    ctx.load(dataclasses.replace(pb, capacity_units=0))
    with pytest.raises(jsv.JsvError):
        ctx.search(D, se.slo_latency_us, se.slo_accuracy, 8)
    # switching the mode off gives the single-tuple search again
    ctx.load(pb)
    ctx.set_mixtures(False)
    try:
        o = oracle.Oracle.from_problem(pb)
        want = o.search(D, se.slo_latency_us, se.slo_accuracy, 0)[0]
        got = ctx.search(D, se.slo_latency_us, se.slo_accuracy, 0)[0]
        for w_, g_ in zip(want, got):
            same(g_, w_)
            assert g_.choice2 == [0xFFFF] * pb.T and g_.replicas2 == [0] * pb.T
    finally:
        ctx.set_mixtures(True)


def test_xr8_full_size_winner_properties(ctx):
    """8 tasks, 240 tuples each, cap 20 (20^8 candidates per level): too large for the oracle's
    search, so the winners are checked for what must hold at any size: every task's option is a
    valid minimal mixture, and cost, latency and accuracy recomputed from the tables (exact
    rationals, tests/pyref.py) are the reported ones and meet the SLOs and S_avail."""
    from fractions import Fraction
    from pyref import PyRef
    w = workloads.xr8()
    pb, se = w.problems[0], w.searches[0]
    ref = PyRef(pb)
    levels = se.demand_mrps[[0, 9, 18, 27, 31, 40]]
    ctx.load(pb)
    res, summ = ctx.search(levels, se.slo_latency_us, se.slo_accuracy, 20)
    assert any(r.feasible for r in res) and not res[-1].feasible
    mixed = 0
    for D, r in zip(levels.tolist(), res):
        if not r.feasible:
            continue
        lat_t, acc_t, cost = [], [], 0
        for t in range(pb.T):
            need = D * int(pb.mult_milli[t])
            c1, c2, m1, m2 = r.choice[t], r.choice2[t], r.replicas[t], r.replicas2[t]
            h1 = 1000 * int(ref.thr[t][c1])
            a1 = ref.accF[t][ref.variant(c1)]
            u1 = int(pb.units[ref.part(c1)])
            if c2 == 0xFFFF:
                assert m2 == 0 and m1 == max(1, -(-need // h1))
                lat_t.append(int(ref.lat[t][c1])); acc_t.append(a1); cost += m1 * u1
            else:
                mixed += 1
                h2 = 1000 * int(ref.thr[t][c2])
                assert c1 < c2 and m1 >= 1 and m2 >= 1
                assert m1 * h1 + m2 * h2 >= need > max((m1 - 1) * h1 + m2 * h2, m1 * h1 + (m2 - 1) * h2)
                lat_t.append(max(int(ref.lat[t][c1]), int(ref.lat[t][c2])))
                acc_t.append((m1 * h1 * a1 + m2 * h2 * ref.accF[t][ref.variant(c2)]) / (m1 * h1 + m2 * h2))
                cost += m1 * u1 + m2 * int(pb.units[ref.part(c2)])
        fin = {}
        for t in ref.order:
            fin[t] = lat_t[t] + max([fin[p] for p in ref.preds[t]], default=0)
        latency = ref.q * max(fin[s] for s in ref.sinks)
        acc = ref._acc_values(acc_t) / ref.amax
        assert (r.cost, r.latency_us) == (cost, latency)
        assert abs(r.accuracy - float(acc)) <= 1e-12 * float(acc)
        assert latency <= se.slo_latency_us and acc >= Fraction(float(se.slo_accuracy)) and cost <= pb.capacity_units
    assert mixed > 0


def crafted(T=2, V=2, P=2, B=1, units=(1, 2), thr=50_000, lat=5000, capacity=20, mult=1000, edges=((0, 1),)):
    """Small problem with regular tables: every tuple serves thr mrps per unit, latencies grow with the tuple id."""
    C = V * P * B
    la = np.zeros((T, V, P, B), dtype=np.uint32)
    th = np.zeros((T, V, P, B), dtype=np.uint32)
    for t in range(T):
        for v in range(V):
            for p in range(P):
                for b in range(B):
                    c = (v * P + p) * B + b
                    la[t, v, p, b] = lat * (1 + c)
                    th[t, v, p, b] = thr * units[p] * (1 + v)
    acc = np.array([[0.6 + 0.3 * v / max(V - 1, 1) for v in range(V)] for _ in range(T)], dtype=np.float64)
    src = np.array([e[0] for e in edges if e[1] < T], dtype=np.uint16)
    dst = np.array([e[1] for e in edges if e[1] < T], dtype=np.uint16)
    return workloads.Problem(T=T, V=V, P=P, B=B, units=np.array(units[:P], dtype=np.uint32),
                             batch=np.array([1 << b for b in range(B)], dtype=np.uint32), latency_us=la, thr_mrps=th,
                             accuracy=acc, src=src, dst=dst, mult_milli=np.array([mult] * T, dtype=np.uint32),
                             capacity_units=capacity, queue_factor=2)


@pytest.mark.parametrize("case", ["one_tuple", "capacity_one", "one_replica", "nothing_fast_enough", "nothing_fits",
                                  "many_replicas"])
def test_edge_cases(ctx, case):
    slo_l, slo_a, D, cap = 400_000, 0.7, [300_000], 16
    if case == "one_tuple":                       # no pair to mix
        pb = crafted(V=1, P=1, units=(1,))
    elif case == "capacity_one":                  # only single replicas of 1-unit tuples fit, and none carries the demand
        pb = crafted(capacity=1)
    elif case == "one_replica":                   # every tuple carries the demand alone: no mixture exists
        pb, D = crafted(), [20_000]
    elif case == "nothing_fast_enough":
        pb, slo_l = crafted(), 1000
    elif case == "nothing_fits":
        pb, D = crafted(capacity=3), [2_000_000]
    else:                                         # hundreds of replicas per tuple, thousands of splits per pair
        pb, D, cap = crafted(thr=1000, capacity=2000, T=1, edges=()), [700_000], 40
    se = workloads.Search(np.array(D, dtype=np.uint32), slo_l, slo_a, cap)
    want = check(ctx, pb, se, cap)
    if case in ("nothing_fast_enough", "nothing_fits", "capacity_one"):
        assert not want[0].feasible
    if case == "one_replica":
        assert want[0].feasible and want[0].choice2 == [0xFFFF] * pb.T


def test_too_many_replicas_is_an_overflow_on_both_sides(ctx):
    pb = crafted(thr=1, capacity=60000, T=1, edges=())           # 1 mrps per unit: 70000 replicas of a tuple alone
    o = oracle.Oracle.from_problem(pb)
    o.set_mixtures(True)
    with pytest.raises(oracle.OracleError) as e:
        o.search([70_000], 400_000, 0.0, 8)
    assert e.value.code == -3
    ctx.load(pb)
    with pytest.raises(jsv.JsvError) as e:
        ctx.search([70_000], 400_000, 0.0, 8)
    assert e.value.code == jsv.E_OVERFLOW
