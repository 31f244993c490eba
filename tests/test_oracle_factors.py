"""Pins of the oracle's per-variant multiplicative factors (Eq. 4, 5): the hand-worked chain,
an independent brute force in exact arithmetic, reduction to fixed factors, and the
invariants of the search over held variants."""
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


def make(g):
    lat = np.array(g["latency_us"], dtype=np.uint32).reshape(g["T"], g["V"], g["P"], g["B"])
    acc = np.array(g["accuracy"], dtype=np.float64)
    return oracle.Oracle(g["T"], g["V"], g["P"], g["B"], g["units"], g["batch"], lat, None, acc,
                         [e[0] for e in g["edges"]], [e[1] for e in g["edges"]], g["mult_milli"], 0,
                         g["queue_factor"])


def test_hand_worked_chain_with_factors(g):
    f = g["factors_eq4_5"]
    o = make(g)
    o.set_factors(f["factor_milli"])
    for s in f["searches"]:
        res, bl, md = o.search([f["demand_mrps"]], s["slo_latency_us"], s["slo_accuracy"], 0)
        r = res[0]
        assert r.feasible and bl == 0 and md == f["demand_mrps"]
        assert (r.index, r.full_index, r.choice, r.cost, r.latency_us, r.replicas) == \
               (s["index"], s["index"], s["choice"], s["cost"], s["latency_us"], s["replicas"])
        assert r.evaluated == 64
        # the replicas are those of the hand-made tables
        va = r.choice[0] // 4
        assert r.replicas[1] == f["replicas_B_by_variant_of_A"][va][r.choice[1]]
    # without factors the second search has another answer (also worked by hand)
    o.set_factors(None)
    s = f["searches"][1]
    r = o.search([f["demand_mrps"]], s["slo_latency_us"], s["slo_accuracy"], 0)[0][0]
    assert (r.index, r.cost) == (s["fixed_factor_answer"]["index"], s["fixed_factor_answer"]["cost"])


def test_hand_worked_objective_with_factors(g):
    f = g["factors_eq4_5"]
    ob = f["objective"]
    o = make(g)
    o.set_factors(f["factor_milli"])
    o.set_objective(1, ob["alpha"], ob["beta"])
    r = o.search([f["demand_mrps"]], ob["slo_latency_us"], ob["slo_accuracy"], 0)[0][0]
    assert (r.index, r.choice, r.cost) == (ob["index"], ob["choice"], ob["cost"])
    assert r.objective == pytest.approx(ob["objective_num"] / ob["objective_den"] - ob["objective_minus"], rel=1e-13)
    # runner-up by hand: pair (1,1), 1 - 0.49
    m = o.objective_margin(f["demand_mrps"], ob["slo_latency_us"], ob["slo_accuracy"], 0)
    assert m == pytest.approx(ob["objective_num"] / ob["objective_den"] - ob["objective_minus"] - 0.51, rel=1e-9)


def tiny(seed):
    """small instance with at least one edge"""
    k = 0
    while True:
        pb, se = workloads.tiny_random(1000 * seed + k)
        if pb.E > 0 and pb.C ** pb.T <= 2500:
            return pb, se
        k += 1


@pytest.mark.parametrize("seed", range(40))
def test_exhaustive_matches_brute_force(seed):
    pb, se = tiny(seed)
    fac = workloads.random_factors(pb, seed)
    o = oracle.Oracle.from_problem(pb)
    o.set_factors(fac)
    ref = PyRef(pb)
    if seed % 3 == 1:
        o.set_search_space(False, True, True); ref.space = (False, True, True)
    if seed % 3 == 2:
        o.set_search_space(True, False, True); ref.space = (True, False, True)
    res, bl, md = o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0)
    best_level = -1
    for l, D in enumerate(se.demand_mrps.tolist()):
        want, count = ref.search_factors(D, se.slo_latency_us, se.slo_accuracy, fac.tolist())
        r = res[l]
        assert r.evaluated == count
        assert bool(r.feasible) == (want is not None)
        if want is None:
            continue
        best_level = l
        full, cost, lat, acc, choice, reps, _ = want
        assert (r.index, r.full_index, r.cost, r.latency_us, r.choice, r.replicas) == \
               (full, full, cost, lat, choice, reps)
        assert r.accuracy == pytest.approx(float(acc), rel=1e-13)
    assert bl == best_level


@pytest.mark.parametrize("seed", range(20))
def test_objective_matches_brute_force(seed):
    pb, se = tiny(100 + seed)
    fac = workloads.random_factors(pb, seed)
    o = oracle.Oracle.from_problem(pb)
    o.set_factors(fac)
    o.set_objective(1, 1.0, 0.035)
    ref = PyRef(pb)
    D = int(se.demand_mrps[0])
    want, _ = ref.search_factors(D, se.slo_latency_us, se.slo_accuracy, fac.tolist(), objective=(1.0, 0.035))
    r = o.search([D], se.slo_latency_us, se.slo_accuracy, 0)[0][0]
    assert bool(r.feasible) == (want is not None)
    if want is None:
        return
    if o.objective_margin(D, se.slo_latency_us, se.slo_accuracy, 0) < 1e-9:
        pytest.skip("two variant combinations tie in the objective within rounding")
    full, cost, lat, acc, choice, reps, obj = want
    assert (r.index, r.cost, r.latency_us, r.choice, r.replicas) == (full, cost, lat, choice, reps)
    assert r.objective == pytest.approx(float(obj), rel=1e-12, abs=1e-12)


@pytest.mark.parametrize("seed", range(12))
def test_whole_constant_factors_reduce_to_fixed_multipliers(seed):
    """If every variant of a task has the same whole-number factor and the multipliers obey
    m_t = sum over predecessors of m_pred * F, both ways of stating the demand agree."""
    pb, se = tiny(200 + seed)
    fac = workloads.random_factors(pb, seed, varying=[], lo=1000, hi=3000, whole=True)
    # multipliers that follow the factors, by a walk in topological order
    preds = {t: [(int(a), e) for e, (a, b) in enumerate(zip(pb.src, pb.dst)) if int(b) == t] for t in range(pb.T)}
    mult, left = {}, set(range(pb.T))
    while left:
        for t in sorted(left):
            if all(a in mult for a, _ in preds[t]):
                mult[t] = int(pb.mult_milli[t]) if not preds[t] else \
                    sum(mult[a] * int(fac[e, 0]) // 1000 for a, e in preds[t])
                left.remove(t)
                break
    pb.mult_milli = np.array([mult[t] for t in range(pb.T)], dtype=np.uint32)
    a = oracle.Oracle.from_problem(pb)
    b = oracle.Oracle.from_problem(pb)
    b.set_factors(fac)
    ra = a.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    rb = b.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    assert ra[1:] == rb[1:]
    for x, y in zip(ra[0], rb[0]):
        assert (x.feasible, x.evaluated, x.flags) == (y.feasible, y.evaluated, y.flags)
        if x.feasible:
            assert (x.full_index, x.cost, x.latency_us, x.choice, x.replicas, x.accuracy) == \
                   (y.full_index, y.cost, y.latency_us, y.choice, y.replicas, y.accuracy)
            assert y.index == y.full_index


@pytest.mark.parametrize("seed", range(25))
def test_exact_prune_keeps_the_optimal_cost(seed):
    """Dropping dominated choices inside every combination of held variants cannot change the
    cheapest feasible cost; thinning can only raise it.  The winner always checks out when
    its demands are recomputed from its own variants."""
    pb, se = tiny(300 + seed)
    fac = workloads.random_factors(pb, seed)
    o = oracle.Oracle.from_problem(pb)
    o.set_factors(fac)
    ref = PyRef(pb)
    cap = max(2 * pb.V, se.prune_cap)
    D = int(se.demand_mrps[-1])
    full = o.search([D], se.slo_latency_us, se.slo_accuracy, 0)[0][0]
    pr = o.search([D], se.slo_latency_us, se.slo_accuracy, cap)[0][0]
    assert pr.evaluated <= full.evaluated
    if pr.feasible:
        assert full.feasible and pr.cost >= full.cost
        need = ref.demands(D, [c // (pb.P * pb.B) for c in pr.choice], fac.tolist())
        reps = [max(1, -(-need[t] // (1000 * int(ref.thr[t][c])))) for t, c in enumerate(pr.choice)]
        assert pr.replicas == reps
        assert pr.cost == sum(r * int(pb.units[ref.part(c)]) for r, c in zip(reps, pr.choice))
        assert pr.latency_us == ref.latency(pr.choice) <= se.slo_latency_us
    if not (pr.flags & 1):
        assert pr.feasible == full.feasible
        if full.feasible:
            assert pr.cost == full.cost


@pytest.mark.parametrize("seed", range(10))
def test_held_combinations_partition_the_space(seed):
    """Only tasks whose outgoing factors differ between variants are held; whichever they
    are, the combinations together cover every candidate exactly once."""
    pb, se = tiny(400 + seed)
    o = oracle.Oracle.from_problem(pb)
    tails = sorted(set(int(a) for a in pb.src))
    for varying in (tails, tails[:1], []):
        o.set_factors(workloads.random_factors(pb, seed, varying=varying))
        # a latency SLO nothing meets: the search only counts
        r = o.search([50_000], 1, 0.0, 0)[0][0]
        assert not r.feasible and r.evaluated == pb.C ** pb.T


def test_argument_errors(g):
    o = make(g)
    with pytest.raises(oracle.OracleError):
        o.set_factors([[0, 1000]])
    with pytest.raises(oracle.OracleError):
        o.set_factors([[1000, 1_000_001]])
    with pytest.raises(ValueError):
        o.set_factors([[1000, 1000, 1000]])
    o.set_factors(g["factors_eq4_5"]["factor_milli"])
    with pytest.raises(oracle.OracleError):
        o.search_range(260000, 100000, 0.5, 0, 0, 10)
    with pytest.raises(oracle.OracleError):
        o.space(260000, 100000, 0)
    o.set_search_space(True, True, False)
    with pytest.raises(oracle.OracleError):
        o.search([260000], 100000, 0.5, 0)
    o.set_search_space(True, True, True)
    # demand beyond the range of the flow arithmetic
    big = make(g)
    big.set_factors([[1_000_000, 1_000_000]])
    with pytest.raises(oracle.OracleError):
        big.search([4_000_000_000], 100000, 0.0, 0)
