"""GPU edge cases: degenerate graphs and spaces, limits, API behaviour."""
import numpy as np
import pytest

import oracle
from paper_2603_08797_amd import jsv, workloads as W
from test_gpu_parity import REL, same, check_search

pytestmark = pytest.mark.gpu
U32 = 2**32 - 1


@pytest.fixture(scope="module")
def ctx():
    j = jsv.Jsv(device=0)
    yield j
    j.close()


def _problem(T, V, P, B, seed, edges, mult=None, capacity=0):
    r = W.SplitMix64(31, seed)
    lat = np.zeros((T, V, P, B), dtype=np.uint32)
    thr = np.zeros((T, V, P, B), dtype=np.uint32)
    for i in np.ndindex(T, V, P, B):
        lat[i] = r.randint(500, 30000)
        thr[i] = r.randint(20_000, 900_000)
    acc = np.sort(0.55 + 0.44 * np.array([[r.uniform() for _ in range(V)] for _ in range(T)]), axis=1)
    return W.Problem(T, V, P, B, np.arange(1, P + 1, dtype=np.uint32),
                     np.array([1 << b for b in range(B)], dtype=np.uint32), lat, thr, acc,
                     np.array([e[0] for e in edges], dtype=np.uint16),
                     np.array([e[1] for e in edges], dtype=np.uint16),
                     np.array(mult if mult else [1000] * T, dtype=np.uint32), capacity, 2)


def _search(D, slo_l, slo_a, cap=0):
    return W.Search(np.array(D, dtype=np.uint32), slo_l, slo_a, cap)


def test_single_task(ctx):
    pb = _problem(1, 3, 4, 3, 1, [])
    check_search(ctx, pb, _search([5000, 90000, 400000], 40000, 0.9))


def test_single_task_maximum_choices(ctx):
    pb = _problem(1, 8, 16, 16, 2, [])          # C = 2048 = JSV_MAX_CHOICES
    check_search(ctx, pb, _search([70000], 50000, 0.8))
    check_search(ctx, pb, _search([70000], 50000, 0.8, cap=64))


def test_sixteen_task_chain_and_wide_graph(ctx):
    T = 16
    chain = _problem(T, 2, 1, 1, 3, [(i, i + 1) for i in range(T - 1)])
    check_search(ctx, chain, _search([30000], 2 * 16 * 30000, 0.0))      # 2^16 candidates
    check_search(ctx, chain, _search([30000], 330000, 0.02))
    # every task isolated: 16 sources that are also sinks
    wide = _problem(T, 2, 1, 1, 4, [], mult=[250 * (1 + t % 4) for t in range(T)])
    check_search(ctx, wide, _search([30000, 900000], 50000, 0.6))
    # reversed labels: task ids against the topological order
    rev = _problem(T, 2, 1, 1, 5, [(i + 1, i) for i in range(T - 1)])
    check_search(ctx, rev, _search([30000], 400000, 0.01))


def test_dense_graph_with_uneven_multipliers(ctx):
    T = 6
    edges = [(i, j) for i in range(T) for j in range(i + 1, T)]
    pb = _problem(T, 2, 2, 2, 6, edges, mult=[1000, 300, 2500, 700, 1200, 450], capacity=40)
    check_search(ctx, pb, _search([20000, 150000, 700000], 150000, 0.35))
    check_search(ctx, pb, _search([20000, 150000], 150000, 0.35, cap=4))


def test_infeasible_is_not_an_error(ctx):
    pb = _problem(3, 2, 2, 2, 7, [(0, 1), (1, 2)])
    ctx.load(pb)
    res, summ = ctx.search([1000], U32, 1.0000001, 0)
    assert not res[0].feasible and res[0].index == 2**64 - 1 and res[0].cost == 2**31 - 1
    assert (summ.best_level, summ.max_demand_mrps) == (-1, 0)
    check_search(ctx, pb, _search([1000], 100, 0.0))               # latency SLO below any path
    # the prune's latency filter empties every list: nothing is evaluated
    res, summ = ctx.search([1000], 100, 0.0, 4)
    ref, _, _ = oracle.Oracle.from_problem(pb).search([1000], 100, 0.0, 4)
    assert res[0].evaluated == 0 == ref[0].evaluated and not res[0].feasible


def test_capacity_bound_is_inclusive_and_binding(ctx):
    pb = _problem(3, 2, 3, 2, 8, [(0, 1), (0, 2)])
    ctx.load(pb)
    free, _ = ctx.search([300000], U32, 0.0, 0)
    c = free[0].cost
    for cap_units, want in ((c, True), (c - 1, False)):
        pb.capacity_units = cap_units
        ctx.load(pb)
        res, _ = ctx.search([300000], U32, 0.0, 0)
        assert res[0].feasible == want
        check_search(ctx, pb, _search([300000], U32, 0.0))


def test_unsorted_and_repeated_demand_levels(ctx):
    pb = _problem(4, 2, 2, 2, 9, [(0, 1), (1, 2), (1, 3)], capacity=14)
    D = [500000, 1000, 90000, 90000, 250000, 1000]
    res, summ = check_search(ctx, pb, _search(D, 120000, 0.3))
    assert res[2] == res[3] and res[1] == res[5]


def test_derived_throughput_equals_explicit_table(ctx):
    w = W.chain3()
    pb, se = w.problems[0], w.searches[0]
    ctx.load(pb)
    a, _ = ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0)
    ctx.load(pb, derive_throughput=True)
    b, _ = ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0)
    assert a == b
    o = oracle.Oracle.from_problem(pb, derive_throughput=True)
    ref, _, _ = o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0, threads=4)
    same(b[0], ref[0])


def test_lent_workspace_too_small_is_reported(ctx):
    pb = W.diamond5().problems[0]
    ctx.load(pb)
    import torch
    t = torch.empty(4096, dtype=torch.uint8, device="cuda")
    p = (t.data_ptr() + 255) // 256 * 256
    assert ctx._lib.jsv_set_workspace(ctx._h, p, 1024) == jsv.OK
    with pytest.raises(jsv.JsvError) as e:
        ctx.search([1000], 100000, 0.5, 40)
    assert e.value.code == jsv.E_WORKSPACE
    ctx._lib.jsv_set_workspace(ctx._h, None, 0)
    ctx.search([1000], 100000, 0.5, 40)


def test_cost_overflow_is_reported(ctx):
    pb = _problem(2, 1, 1, 1, 10, [(0, 1)])
    pb.thr_mrps[:] = 1
    pb.units[:] = 4000
    ctx.load(pb)
    with pytest.raises(jsv.JsvError) as e:
        ctx.search([4_000_000_000], U32, 0.0, 0)       # 4e9 replicas x 4000 units
    assert e.value.code == jsv.E_OVERFLOW


def test_repeated_runs_and_a_second_context_agree(ctx):
    w = W.diamond5()
    pb, se = w.problems[0], w.searches[0]
    ctx.load(pb)
    a, _ = ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    b, _ = ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    import torch
    other = jsv.Jsv(device=0, stream=torch.cuda.Stream())
    other.load(pb)
    c, _ = other.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    other.close()
    assert a == b == c


def test_pruned_cost_matches_exhaustive_cost_when_nothing_was_thinned(ctx):
    w = W.chain3()
    pb, se = w.problems[0], w.searches[0]
    ctx.load(pb)
    full, _ = ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0)
    pr, _ = ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, pb.C)
    assert pr[0].flags & 1 == 0 and pr[0].evaluated < full[0].evaluated
    assert (pr[0].feasible, pr[0].cost) == (full[0].feasible, full[0].cost)


def test_large_costs_take_the_64_bit_key_path(ctx):
    """Costs of ~1e7 units per task do not fit the 32-bit local key (cost bits + rank
    bits > 31), so the enumeration falls back to comparing full 64-bit keys."""
    pb = _problem(3, 2, 3, 4, 11, [(0, 1), (1, 2)])
    pb.thr_mrps[:] = (pb.thr_mrps % 8) + 8              # 8..15 mrps per replica: ~3e8 replicas
    pb.units[:] = 1
    res, _ = check_search(ctx, pb, _search([3_000_000_000], 120000, 0.5))
    assert res[0].flags & 2 and res[0].feasible and res[0].cost > 2**29
    res, _ = check_search(ctx, pb, _search([3_000_000_000, 1000], 120000, 0.5))
    assert [r.flags & 2 for r in res] == [2, 0]          # the small level fits the fast path
    check_search(ctx, pb, _search([3_000_000_000, 2_000_000_000, 1000], 120000, 0.5, cap=8))


def test_equal_latencies_inside_a_variant_keep_the_lowest_index(ctx):
    """All choices of a variant share one latency and one cost: every tie must go to the
    lowest candidate index although the kernel walks a variant in latency order."""
    pb = _problem(3, 2, 2, 3, 12, [(0, 1), (0, 2)])
    pb.latency_us[:, 0] = 7000
    pb.latency_us[:, 1] = 9000
    pb.thr_mrps[:] = 500_000
    pb.units[:] = 2
    check_search(ctx, pb, _search([100000, 1_400_000], 60000, 0.0))
    check_search(ctx, pb, _search([100000], 60000, 0.9))


def test_many_variants_few_choices_each(ctx):
    """P = B = 1: every stream group holds one choice and three padding entries."""
    pb = _problem(3, 12, 1, 1, 13, [(0, 1), (1, 2)])
    check_search(ctx, pb, _search([40000, 600000], 70000, 0.55))
    check_search(ctx, pb, _search([40000], 70000, 0.55, cap=24))


def test_source_tasks_after_the_first_position(ctx):
    """Two extra sources feeding one sink: positions 1 and 2 are sources too."""
    pb = _problem(4, 2, 2, 2, 14, [(0, 3), (1, 3), (2, 3)], mult=[1000, 400, 1600, 1000])
    check_search(ctx, pb, _search([50000, 300000], 90000, 0.4))
    wide = _problem(3, 3, 2, 2, 15, [])                  # three isolated tasks
    check_search(ctx, wide, _search([50000], 50000, 0.7))


def test_three_in_lane_positions_with_both_key_widths(ctx):
    """Many levels of a 6-task graph with 12 choices per task: enough lanes for the planner to
    loop three (resp. two) positions inside a lane; huge demands force the 64-bit keys,
    small ones run the 32-bit fast path, in one sweep."""
    edges = [(0, 1), (0, 2), (1, 3), (2, 3), (3, 4), (1, 5)]
    pb = _problem(6, 2, 3, 2, 16, edges, mult=[1000, 700, 1300, 1000, 1000, 400])
    pb.thr_mrps[:] = (pb.thr_mrps % 8) + 8
    pb.units[:] = 1
    big = [2_000_000_000 + 7_000_000 * k for k in range(40)]
    small = [1000 + 37 * k for k in range(24)]
    res, _ = check_search(ctx, pb, _search(big + small, 200000, 0.45))
    assert all(r.flags & 2 for r in res[:40]) and not any(r.flags & 2 for r in res[40:])
    assert any(r.feasible for r in res)
    five = _problem(5, 2, 3, 2, 17, [(0, 1), (1, 2), (2, 3), (3, 4)])
    five.thr_mrps[:] = (five.thr_mrps % 8) + 8
    five.units[:] = 1
    check_search(ctx, five, _search(big + small, 200000, 0.3))
    ctx.set_objective(1, 1.0, 1e-9)
    try:
        ctx.load(pb)
        got, _ = ctx.search(big[:8] + small[:8], 200000, 0.45, 0)
    finally:
        ctx.set_objective(0)
    o = oracle.Oracle.from_problem(pb)
    o.set_objective(1, 1.0, 1e-9)
    ref, _, _ = o.search(big[:8] + small[:8], 200000, 0.45, 0, threads=16)
    for a, b in zip(got, ref):
        assert a.feasible == b.feasible
        if b.feasible:
            assert abs(a.objective - b.objective) <= 1e-12
            if a.index != b.index:      # only an objective tie between different variants may differ
                assert a.objective == pytest.approx(b.objective, abs=1e-12)
            else:
                same(a, b)


@pytest.mark.parametrize("name", ["diamond5", "xr8", "chain3"])
def test_threshold_of_exactly_one_accepts_the_most_accurate_assignment(ctx, name):
    """SLO_a = 1.0 (no accuracy loss allowed): A_max and every candidate's A_raw are formed by
    one order of operations, so the all-best-variant candidates pass Eq. 13 on the device as
    they do in the oracle; on graphs whose source has several successors a different
    summation order would land one ulp below A_max and reject them."""
    w = W.BENCH_WORKLOADS[name](seed=0)
    pb, se = w.problems[0], w.searches[0]
    o = oracle.Oracle.from_problem(pb)
    dem = se.demand_mrps[:6:2] if len(se.demand_mrps) > 1 else se.demand_mrps
    cap = 10 if name == "xr8" else se.prune_cap
    slo_l = se.slo_latency_us * (2 if name == "chain3" else 1)   # the best variants are the slowest
    ctx.load(pb)
    res, summ = ctx.search(dem, slo_l, 1.0, cap)
    ref, bl, md = o.search(dem, slo_l, 1.0, cap, threads=16)
    assert any(b.feasible for b in ref)
    for l, (a, b) in enumerate(zip(res, ref)):
        same(a, b, f"{name} level {l}")
        if b.feasible:
            assert a.accuracy == 1.0
            assert all(c // (pb.P * pb.B) == int(np.argmax(pb.accuracy[t])) for t, c in enumerate(a.choice))
    assert (summ.best_level, summ.max_demand_mrps) == (bl, md)
    # all candidates of the first level that the oracle accepts, the device accepts, and vice versa
    D = int(dem[0])
    K, space, _ = o.space(D, slo_l, cap)
    idx = np.random.default_rng(3).integers(0, space, size=200_000, dtype=np.uint64)
    idx[0] = ref[0].index if ref[0].feasible else 0
    ga = ctx.eval_candidates(D, slo_l, 1.0, cap, idx)
    gb = o.eval(D, slo_l, 1.0, cap, idx)
    assert np.array_equal(ga[4], gb[4]) and (gb[4] & 2).any()


@pytest.mark.parametrize("seed", range(30))
def test_threshold_of_exactly_one_on_random_graphs(ctx, seed):
    """Random multi-branch graphs with uneven multipliers: shares like 1/3 and 3/7 make the
    weighted sums inexact, which is where summation order shows."""
    r = W.SplitMix64(77, seed)
    T = 4 + seed % 4
    edges = [(a, b) for a in range(T) for b in range(a + 1, T) if r.uniform() < 0.55]
    mult = [int(r.randint(300, 1700)) for _ in range(T)]
    pb = _problem(T, 3, 2, 2, 100 + seed, edges, mult=mult)
    check_search(ctx, pb, _search([20000, 250000], 400000, 1.0))
    check_search(ctx, pb, _search([20000], 400000, 1.0, cap=6))


@pytest.mark.parametrize("name,cap", [("diamond5", 40), ("xr8", 10), ("chain4", 0)])
def test_results_do_not_depend_on_the_launch_geometry(ctx, name, cap):
    """1, 3 and 8 blocks per compute unit; half, double and eight times the lanes the planner
    aims for (which changes how many tasks a lane loops over and the tile cut); bounds on and
    off; both objective modes: every field of every record is the same."""
    w = W.BENCH_WORKLOADS[name](seed=0)
    pb, se = w.problems[0], w.searches[0]
    dem = se.demand_mrps[::7] if len(se.demand_mrps) > 1 else se.demand_mrps
    ctx.load(pb)
    try:
        for objective in (0, 1):
            ctx.set_objective(objective, 1.0, 0.035)
            ctx.set_geometry(0, 0)
            ctx.set_bounds(True)
            want, wsum = ctx.search(dem, se.slo_latency_us, se.slo_accuracy, cap)
            for bounds in (False, True):
                ctx.set_bounds(bounds)
                for blocks, lanes in ((1, 100), (3, 100), (8, 100), (0, 50), (0, 200), (2, 800), (0, 12)):
                    ctx.set_geometry(blocks, lanes)
                    got, gsum = ctx.search(dem, se.slo_latency_us, se.slo_accuracy, cap)
                    assert got == want, (name, objective, bounds, blocks, lanes)
                    assert (gsum.best_level, gsum.max_demand_mrps) == (wsum.best_level, wsum.max_demand_mrps)
    finally:
        ctx.set_geometry(0, 0)
        ctx.set_bounds(True)
        ctx.set_objective(0)
    with pytest.raises(jsv.JsvError) as e:
        ctx.set_geometry(9, 0)
    assert e.value.code == jsv.E_BADARG


# ---- the loop that keeps one accuracy mask per variant of the innermost position ---------------
# It runs where a lane loops over two or three positions.  Small graphs get there when the planner
# is asked for few lanes (one block per compute unit, 1 % of the usual lane count); every case
# also runs with the automatic geometry.
GEOMETRIES = [(0, 0), (1, 1), (2, 4)]


def _check_under_geometries(ctx, pb, se, bounds=(True, False)):
    try:
        for blocks, lanes in GEOMETRIES:
            ctx.set_geometry(blocks, lanes)
            for b in bounds:
                ctx.set_bounds(b)
                check_search(ctx, pb, se)
    finally:
        ctx.set_geometry(0, 0)
        ctx.set_bounds(True)


@pytest.mark.parametrize("V", [1, 2, 7, 8, 9])
def test_variant_counts_around_the_limit_of_the_masked_loop(ctx, V):
    """Up to eight variants in the innermost position's stream take the loop with one mask per
    variant; nine take the general loop.  Same answers either way (oracle), with and without
    bounds and in objective mode."""
    T = 7 if V == 1 else 5               # (few choices per task need more tasks for a lane to loop over two)
    edges = [(0, 1), (0, 2), (1, 3), (2, 3), (3, 4)] + ([(2, 5), (4, 6)] if V == 1 else [])
    pb = _problem(T, V, 2, 2, 40 + V, edges, capacity=60)
    se = _search([30000, 150000, 700000], 160000 if V > 1 else 260000, 0.6)
    _check_under_geometries(ctx, pb, se)
    o = oracle.Oracle.from_problem(pb)
    o.set_objective(1, 1.0, 0.02)
    ref, _, _ = o.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0, threads=16)
    margins = [o.objective_margin(int(D), se.slo_latency_us, se.slo_accuracy, 0) if V <= 2 else None
               for D in se.demand_mrps]
    ctx.set_objective(1, 1.0, 0.02)
    try:
        ctx.load(pb)
        for blocks, lanes in GEOMETRIES:
            ctx.set_geometry(blocks, lanes)
            got, _ = ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 0)
            for l, (a, b) in enumerate(zip(got, ref)):
                assert a.feasible == b.feasible
                if not b.feasible:
                    continue
                assert abs(a.objective - b.objective) <= 1e-12 * max(1.0, abs(b.objective))
                if a.index == b.index or (margins[l] is not None and margins[l] > 1e-9):
                    same(a, b, f"level {l}")
    finally:
        ctx.set_objective(0)
        ctx.set_geometry(0, 0)


@pytest.mark.parametrize("PB", [(1, 1), (1, 2), (1, 3), (1, 5), (2, 3), (1, 7), (3, 3)])
def test_every_length_of_a_run_of_equal_accuracy(ctx, PB):
    """The second in-lane position goes through the stream four digits at a time, then two, then
    one: runs of 1, 2, 3, 5, 6, 7 and 9 digits per variant cover every remainder."""
    P, B = PB
    K = 3 * P * B
    T = 10 if K <= 3 else 6 if K <= 9 else 5
    edges = [(0, 1), (1, 2), (0, 3), (3, 4)] + ([(2, 5)] if T >= 6 else []) + ([(4, 6), (5, 7), (6, 8), (7, 9)] if T == 10 else [])
    pb = _problem(T, 3, P, B, 60 + 10 * P + B, edges, capacity=0)
    for slo_a in (0.0, 0.62, 0.8):
        _check_under_geometries(ctx, pb, _search([20000, 400000], 250000 if K > 3 else 1200000, slo_a))


def test_variants_of_equal_accuracy_share_their_run(ctx):
    """Two variants of a task with bit-identical accuracy: in the second position they form one
    run, in the innermost they keep their own masks, which are then equal."""
    pb = _problem(5, 4, 2, 2, 77, [(0, 1), (1, 2), (2, 3), (0, 4)])
    pb.accuracy[:, 1] = pb.accuracy[:, 2]
    for slo_a in (0.55, 0.7, 0.85):
        _check_under_geometries(ctx, pb, _search([50000, 900000], 210000, slo_a))


def test_long_streams_and_long_runs_in_the_masked_loop(ctx):
    """512 choices per task in 8 variants: 128 records in the innermost stream, runs of 64 digits in
    the second position."""
    pb = _problem(3, 8, 8, 8, 91, [(0, 1), (0, 2)], capacity=0)
    _check_under_geometries(ctx, pb, _search([60000, 2_000_000], 140000, 0.7), bounds=(True,))
    _check_under_geometries(ctx, pb, _search([60000], 140000, 0.7, cap=96), bounds=(False,))


# ---- three in-lane positions with the pair stream -----------------------------------------------
# Cost modes, single tuples, at most eight variants in the innermost position, four or more digits
# of the third position per tile: the digits of the third position are the slots, the stream holds
# (second position, innermost position) pairs.  Few lanes asked of the planner bring small graphs there.
PAIR_SHAPES = {
    # position 1 a successor of position 0 (chain), a source (two sources), position 2 a source, both
    "chain": [(0, 1), (1, 2), (2, 3), (3, 4)],
    "source_at_1": [(0, 2), (1, 2), (2, 3), (3, 4)],
    "source_at_2": [(0, 1), (2, 3), (1, 4), (3, 4)],
    "sources_at_1_and_2": [(0, 3), (1, 3), (2, 4), (3, 4)],
    "fan": [(0, 1), (0, 2), (1, 3), (2, 3), (0, 4)],
}


@pytest.mark.parametrize("shape", sorted(PAIR_SHAPES))
@pytest.mark.parametrize("PB", [(1, 5), (2, 3), (1, 7), (3, 3)])
def test_pair_stream_with_every_remainder_of_a_run(ctx, shape, PB):
    """Runs of 5, 6, 7 and 9 digits per variant of the third position: batches of four slots and
    every remainder (1, 2, 3), cut further by the tiles' chunks; the second position a successor
    of the innermost one or a source; with and without bounds; thresholds that no, some and
    most variant combinations meet."""
    P, B = PB
    pb = _problem(5, 3, P, B, 300 + 10 * P + B, PAIR_SHAPES[shape], mult=[1000, 800, 1200, 1000, 900], capacity=0)
    try:
        for blocks, lanes in ((1, 1), (1, 3), (0, 0)):
            ctx.set_geometry(blocks, lanes)
            for b in (False, True):
                ctx.set_bounds(b)
                for slo_a in (0.0, 0.66, 0.8):
                    check_search(ctx, pb, _search([20000, 600000], 240000, slo_a))
    finally:
        ctx.set_geometry(0, 0)
        ctx.set_bounds(True)


def test_pair_stream_with_capacity_and_thinned_lists(ctx):
    """A capacity that binds (the cost bound of the bounded search moves) and a prune cap that thins
    the lists to uneven runs, on a six-task graph under the small-lane geometries."""
    edges = [(0, 1), (0, 2), (1, 3), (2, 3), (3, 4), (1, 5)]
    pb = _problem(6, 4, 3, 3, 411, edges, mult=[1000, 700, 1300, 1000, 1000, 400], capacity=90)
    try:
        for blocks, lanes in ((1, 1), (2, 2), (0, 0)):
            ctx.set_geometry(blocks, lanes)
            for b in (False, True):
                ctx.set_bounds(b)
                check_search(ctx, pb, _search([15000, 120000, 900000], 300000, 0.6, cap=14))
                check_search(ctx, pb, _search([15000, 120000], 300000, 0.7, cap=22))
    finally:
        ctx.set_geometry(0, 0)
        ctx.set_bounds(True)


def test_pair_stream_with_full_records_in_both_objective_modes(ctx):
    """Six tasks from the benchmark's table generator (5 variants of 48 choices, cap 20): every list
    thins to four survivors per variant, so every record of the innermost stream is full and every
    run of the other positions has four digits - the shape of the 8-task sweep, small enough for
    the oracle to go through whole levels.  Cost mode and Eq. 14, with and without bounds, under
    geometries that give three in-lane positions with tiles of four and more digits."""
    sizes, batches = list(range(1, 9)), [1, 2, 4, 8, 16, 32]
    lat, thr, acc = W._tables(W.SplitMix64(905, 1), W.SplitMix64(905, 2), 6, 5, sizes, 8, batches)
    edges = [(0, 1), (0, 2), (0, 3), (1, 4), (2, 4), (3, 4), (4, 5)]
    pb = W._problem(6, 5, sizes, 8, batches, lat, thr, acc, edges, [1000, 1000, 900, 1100, 1000, 1000], 64)
    dem = [30000, 80000, 150000, 600000]
    slo_l, slo_a, cap = 220000, 0.5, 20
    o = oracle.Oracle.from_problem(pb)
    assert o.accuracy_margin(slo_a) > 1e-9
    for D in dem:
        K, space, thinned = o.space(D, slo_l, cap)
        assert list(K) == [20] * 6 and thinned, K        # four per variant everywhere
    ref_cost, _, _ = o.search(dem, slo_l, slo_a, cap, threads=16)
    o.set_objective(1, 1.0, 0.035)
    ref_obj, _, _ = o.search(dem, slo_l, slo_a, cap, threads=16)
    assert sum(r.feasible for r in ref_cost) >= 2 and not all(r.feasible for r in ref_cost)
    try:
        for blocks, lanes in ((0, 5), (1, 3), (0, 0)):
            ctx.set_geometry(blocks, lanes)
            for b in (False, True):
                ctx.set_bounds(b)
                ctx.set_objective(0)
                ctx.load(pb)
                got, _ = ctx.search(dem, slo_l, slo_a, cap)
                for l, (x, y) in enumerate(zip(got, ref_cost)):
                    same(x, y, f"cost mode, geometry {blocks},{lanes}, bounds {b}, level {l}")
                ctx.set_objective(1, 1.0, 0.035)
                got, _ = ctx.search(dem, slo_l, slo_a, cap)
                for l, (x, y) in enumerate(zip(got, ref_obj)):
                    where = f"objective mode, geometry {blocks},{lanes}, bounds {b}, level {l}"
                    assert x.feasible == y.feasible, where
                    if not y.feasible:
                        continue
                    assert abs(x.objective - y.objective) <= 1e-12 * max(1.0, abs(y.objective)), where
                    if x.index == y.index:
                        same(x, y, where)
                    else:       # only candidates of different variants within rounding of each other may swap
                        assert abs(x.objective - y.objective) <= 1e-9, where
                        assert [c // 48 for c in x.choice] != [c // 48 for c in y.choice], where
    finally:
        ctx.set_objective(0)
        ctx.set_geometry(0, 0)
        ctx.set_bounds(True)
