"""The latency / capacity bounds of the enumeration change what the kernel skips, never the
result: every search is run with bounds on and off and compared field by field."""
import dataclasses

import numpy as np
import pytest

from paper_2603_08797_amd import jsv, workloads

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    j = jsv.Jsv(device=0)
    yield j
    j.set_bounds(True)
    j.close()


def both(ctx, run, mixtures=False):
    ctx.set_bounds(True)
    a, sa = run()
    ctx.set_bounds(False)
    b, sb = run()
    ctx.set_bounds(True)
    assert len(a) == len(b)
    for x, y in zip(a, b):
        assert dataclasses.asdict(x) == dataclasses.asdict(y)
    assert (sa.best_level, sa.max_demand_mrps) == (sb.best_level, sb.max_demand_mrps)
    # off, or too few tiles for bounds to pay: every candidate's tests are issued;
    # on: counted per wave and per padded quad
    total = sum(r.evaluated for r in b)
    if mixtures:
        # the latency-sorted stream of options is left early with and without bounds, so the count is
        # per wave and padded quad in both runs; bounds only ever take candidates away
        assert sa.candidates_visited <= sb.candidates_visited
    else:
        assert sb.candidates_visited == total
    return sa.candidates_visited, sb.candidates_visited, total


@pytest.mark.parametrize("name", ["chain3", "diamond5", "chain4"])
def test_bench_workloads(ctx, name):
    w = workloads.BENCH_WORKLOADS[name]()
    pb, se = w.problems[0], w.searches[0]
    ctx.load(pb)
    both(ctx, lambda: ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap))


def test_xr8_small_cap_cuts_most_of_the_sweep(ctx):
    w = workloads.xr8(prune_cap=15)
    pb, se = w.problems[0], w.searches[0]
    ctx.load(pb)
    on, off, total = both(ctx, lambda: ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 15))
    assert on < off // 2          # the upper half of the sweep cannot fit S_avail, the lower half has cheap answers


def test_xr8_at_the_benchmark_size(ctx):
    """cap 20 (20^8 candidates per level), the configuration bench.py times: a few levels from
    both sides of the feasibility edge, plain enumeration against the bounded search."""
    w = workloads.xr8()
    pb, se = w.problems[0], w.searches[0]
    levels = se.demand_mrps[[0, 13, 26, 31, 32, 45, 63]]
    ctx.load(pb)
    on, off, total = both(ctx, lambda: ctx.search(levels, se.slo_latency_us, se.slo_accuracy, se.prune_cap))
    assert total == 7 * 20 ** 8 and on < off // 4


@pytest.mark.parametrize("seed", [1, 2, 3])
def test_first_bound_from_the_plan_kernel(ctx, seed):
    """An instance with at least eight tiles per block of the grid starts from the cost of a
    candidate that the plan kernel reaches by descent, not from S_avail: the other seeds of xr8 at
    the benchmark size, and thinner lists with one block per compute unit (whose tiles still
    outnumber that grid eight to one), plain enumeration against the bounded search."""
    w = workloads.xr8(seed=seed)
    pb, se = w.problems[0], w.searches[0]
    levels = se.demand_mrps[[0, 9, 18, 27, 36]]
    ctx.load(pb)
    on, off, total = both(ctx, lambda: ctx.search(levels, se.slo_latency_us, se.slo_accuracy, se.prune_cap))
    assert total == 5 * 20 ** 8 and on < off // 4
    ctx.set_geometry(1, 0)
    try:
        on, off, total = both(ctx, lambda: ctx.search(levels, se.slo_latency_us, se.slo_accuracy, 14))
        assert on < off
    finally:
        ctx.set_geometry(0, 0)


@pytest.mark.parametrize("seed", range(40))
def test_tiny_random(ctx, seed):
    pb, se = workloads.tiny_random(9000 + seed)
    ctx.load(pb)
    both(ctx, lambda: ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap))
    ctx.set_objective(1, 1.0, 0.035)
    try:
        both(ctx, lambda: ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap))
    finally:
        ctx.set_objective(0, 1.0, 0.035)


def test_batch(ctx):
    w = workloads.dagbatch(n=48)
    ctx.load_batch(w.problems, w.searches)
    both(ctx, ctx.search_loaded_batch)


@pytest.mark.parametrize("seed", range(12))
def test_mixtures(ctx, seed):
    pb, se = workloads.tiny_mixture(9100 + seed)
    if pb.capacity_units == 0:
        pb = dataclasses.replace(pb, capacity_units=30)
    ctx.load(pb)
    ctx.set_mixtures(True)
    try:
        both(ctx, lambda: ctx.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 9), mixtures=True)
    finally:
        ctx.set_mixtures(False)


def test_first_bound_over_mixtures(ctx):
    """The plan kernel's first bound with two tuples per task: xr8 at cap 14 with one block per
    compute unit (the instance's tiles outnumber that grid eight to one), a few levels, bounds on
    and off."""
    w = workloads.xr8()
    pb, se = w.problems[0], w.searches[0]
    levels = se.demand_mrps[[0, 12, 24, 31]]
    ctx.load(pb)
    ctx.set_mixtures(True)
    ctx.set_geometry(1, 0)
    try:
        on, off, total = both(ctx, lambda: ctx.search(levels, se.slo_latency_us, se.slo_accuracy, 14), mixtures=True)
        assert on < off
    finally:
        ctx.set_geometry(0, 0)
        ctx.set_mixtures(False)
