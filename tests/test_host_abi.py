"""Host side of the C ABI without a GPU: the library loads, exports every symbol
declared in include/jsv.h, and rejects bad input with the documented codes."""
import os
import re

import numpy as np
import pytest

from paper_2603_08797_amd import jsv, workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_every_declared_symbol_is_exported():
    with open(os.path.join(ROOT, "include", "jsv.h")) as f:
        declared = re.findall(r"JSV_API\s+[\w\s\*]+?\b(jsv_\w+)\s*\(", f.read())
    assert sorted(declared) == sorted(jsv.EXPORTS)
    lib = jsv.load_library()
    for name in declared:
        assert getattr(lib, name) is not None


def test_struct_sizes_match_the_header():
    import ctypes
    assert ctypes.sizeof(jsv.JsvResult) == 8 * 4 + 4 * 4 + 2 * 16 + 4 * 16 + 8 + 2 * 16 + 4 * 16
    assert ctypes.sizeof(jsv.JsvSummary) == 32


def test_a_fresh_plan_has_every_mode_switch_off(tmp_path):
    """The kernels' argument block (jsv::Plan): default-constructed over memory full of ones,
    every switch reads 0 and every pointer null."""
    import subprocess
    exe = str(tmp_path / "plan_defaults")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-Wall", os.path.join(ROOT, "tests", "c_abi", "plan_defaults.cpp"),
                           "-o", exe])
    out = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert out.returncode == 0 and "plan defaults ok" in out.stdout, out.stdout + out.stderr


def test_reciprocal_division_of_the_tile_set_up(tmp_path):
    """jsv::div_by_magic (how a lane splits its combination into digits) equals / and % for every
    list length, on boundary and random dividends."""
    import subprocess
    exe = str(tmp_path / "div_by_magic")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-Wall", os.path.join(ROOT, "tests", "c_abi", "div_by_magic.cpp"),
                           "-o", exe])
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0 and "div by magic ok" in out.stdout, out.stdout + out.stderr


@pytest.fixture()
def ctx():
    j = jsv.Jsv(use_torch=False)
    yield j
    j.close()


def code(fn, *a, **k):
    with pytest.raises(jsv.JsvError) as e:
        fn(*a, **k)
    return e.value.code


def test_profile_validation(ctx):
    pb, _ = W.tiny_random(1, T=3)
    ok = (pb.T, pb.V, pb.P, pb.B, pb.units, pb.batch, pb.latency_us, pb.thr_mrps, pb.accuracy)
    ctx.load_profile(*ok)
    assert code(ctx.load_profile, 0, *ok[1:]) == jsv.E_BADARG
    assert code(ctx.load_profile, 17, *ok[1:]) == jsv.E_BADARG
    bad = pb.latency_us.copy(); bad.flat[0] = 0
    assert code(ctx.load_profile, *ok[:6], bad, pb.thr_mrps, pb.accuracy) == jsv.E_BADARG
    bad = pb.thr_mrps.copy(); bad.flat[-1] = 0
    assert code(ctx.load_profile, *ok[:6], pb.latency_us, bad, pb.accuracy) == jsv.E_BADARG
    for v in (0.0, 1.5, float("nan")):
        bad = pb.accuracy.copy(); bad[0, 0] = v
        assert code(ctx.load_profile, *ok[:8], bad) == jsv.E_BADARG
    assert code(ctx.load_profile, 1, 64, 8, 8, np.ones(8), np.ones(8), np.ones((1, 64, 8, 8)),
                None, np.ones((1, 64))) == jsv.E_BADARG            # V*P*B > JSV_MAX_CHOICES
    lat1 = np.ones_like(pb.latency_us)                             # 1 us at batch 8 -> 8e9 mrps
    assert code(ctx.load_profile, pb.T, pb.V, pb.P, pb.B, pb.units, np.full(pb.B, 8), lat1, None,
                pb.accuracy) == jsv.E_OVERFLOW


def test_graph_validation(ctx):
    pb, _ = W.tiny_random(1, T=3)
    ctx.load_profile(pb.T, pb.V, pb.P, pb.B, pb.units, pb.batch, pb.latency_us, pb.thr_mrps, pb.accuracy)
    m = [1000, 1000, 1000]
    ctx.set_dag(3, [0, 1], [1, 2], m, 0, 2)
    assert code(ctx.set_dag, 3, [0, 1, 2], [1, 2, 0], m, 0, 2) == jsv.E_CYCLE
    assert code(ctx.set_dag, 3, [0], [0], m, 0, 2) == jsv.E_BADARG          # self loop
    assert code(ctx.set_dag, 3, [0, 0], [1, 1], m, 0, 2) == jsv.E_BADARG    # duplicate edge
    assert code(ctx.set_dag, 3, [0], [3], m, 0, 2) == jsv.E_BADARG          # endpoint out of range
    assert code(ctx.set_dag, 3, [0], [1], [1000, 0, 1000], 0, 2) == jsv.E_BADARG
    assert code(ctx.set_dag, 3, [0], [1], m, 0, 0) == jsv.E_BADARG          # queue factor 0
    assert code(ctx.set_dag, 4, [0], [1], m + [1000], 0, 2) == jsv.E_STATE  # T differs from profile


def test_latency_range_overflow(ctx):
    lat = np.full((2, 1, 1, 1), 2**31, dtype=np.uint32)
    ctx.load_profile(2, 1, 1, 1, [1], [1], lat, np.ones((2, 1, 1, 1)), np.ones((2, 1)))
    assert code(ctx.set_dag, 2, [0], [1], [1000, 1000], 0, 2) == jsv.E_OVERFLOW


def test_search_argument_and_state_errors(ctx):
    assert code(ctx.search, [1000], 1000, 0.5, 0) == jsv.E_STATE            # nothing loaded
    pb, _ = W.tiny_random(1, T=3)
    ctx.load_profile(pb.T, pb.V, pb.P, pb.B, pb.units, pb.batch, pb.latency_us, pb.thr_mrps, pb.accuracy)
    assert code(ctx.search, [1000], 1000, 0.5, 0) == jsv.E_STATE            # no graph yet
    ctx.set_dag(3, [0, 1], [1, 2], [1000] * 3, 0, 2)
    assert code(ctx.search, [], 1000, 0.5, 0) == jsv.E_BADARG
    assert code(ctx.search, [1000, 0], 1000, 0.5, 0) == jsv.E_BADARG
    assert code(ctx.search, [1000], 1000, float("nan"), 0) == jsv.E_BADARG
    assert code(ctx.search, [1000], 1000, 0.5, 2 * pb.V - 1) == jsv.E_BADARG
    assert code(ctx.get_pruned, 1000, 1000, 0, 3) == jsv.E_BADARG           # task out of range


def test_objective_arguments(ctx):
    ctx.set_objective(1, 1.0, 0.035)
    ctx.set_objective(0)
    assert code(ctx.set_objective, 2, 1.0, 0.035) == jsv.E_BADARG
    assert code(ctx.set_objective, 1, -1.0, 0.035) == jsv.E_BADARG
    assert code(ctx.set_objective, 1, 1.0, float("nan")) == jsv.E_BADARG
    assert code(ctx.set_objective, 1, float("inf"), 0.0) == jsv.E_BADARG


def test_workspace_size_and_alignment(ctx):
    pb = W.xr8().problems[0]
    ctx.load(pb)
    a, b = ctx.workspace_bytes(1, 20), ctx.workspace_bytes(64, 20)
    assert 0 < a < b and b % 256 == 0
    lib = jsv.load_library()
    assert lib.jsv_set_workspace(ctx._h, 0x1001, 1 << 20) == jsv.E_BADARG
    assert lib.jsv_set_workspace(ctx._h, None, 0) == jsv.OK


def test_batch_validation_reports_the_offending_problem(ctx):
    w = W.dagbatch(n=6)
    w.problems[4].src = np.array([0, 1], dtype=np.uint16)
    w.problems[4].dst = np.array([1, 0], dtype=np.uint16)
    with pytest.raises(jsv.JsvError) as e:
        ctx.load_batch(w.problems, w.searches)
    assert e.value.code == jsv.E_CYCLE and "problem 4" in str(e.value)


def test_factor_arguments_and_state(ctx):
    pb, _ = W.tiny_random(1, T=3)
    assert code(ctx.set_factors, None) == jsv.E_STATE                        # nothing loaded
    ctx.load_profile(pb.T, pb.V, pb.P, pb.B, pb.units, pb.batch, pb.latency_us, pb.thr_mrps, pb.accuracy)
    ctx.set_dag(3, [], [], [1000] * 3, 0, 2)
    ctx.E = 0
    with pytest.raises(ValueError):
        ctx.set_factors(np.ones((1, pb.V)))                                  # shape must be [E][V]
    lib = jsv.load_library()
    one = np.full((1, pb.V), 1000, dtype=np.uint32)
    assert lib.jsv_set_factors(ctx._h, one.ctypes.data) == jsv.E_BADARG      # a graph without edges
    ctx.set_dag(3, [0, 1], [1, 2], [1000] * 3, 0, 2)
    f = np.full((2, pb.V), 1500, dtype=np.uint32)
    ctx.set_factors(f)
    for bad in (0, 1_000_001):
        g = f.copy(); g[1, 0] = bad
        assert code(ctx.set_factors, g) == jsv.E_BADARG
    ctx.set_factors(None)
    # the full index must fit 64 bits
    big = W.xr8().problems[0]                                                # 240^8 < 2^64: accepted
    ctx.load(big)
    ctx.set_factors(np.full((big.E, big.V), 1000, dtype=np.uint32))
    wide = np.ones((16, 2, 32, 32), dtype=np.uint32)                         # 2048^16 candidates
    ctx.load_profile(16, 2, 32, 32, np.ones(32), np.ones(32), wide * 1000, wide * 1000, np.full((16, 2), 0.9))
    ctx.set_dag(16, [0], [1], [1000] * 16, 0, 2)
    assert code(ctx.set_factors, np.full((1, 2), 1000, dtype=np.uint32)) == jsv.E_OVERFLOW


def test_mode_switches_need_no_device(ctx):
    ctx.set_bounds(False)
    ctx.set_bounds(True)
    ctx.set_mixtures(True)
    pb, se = W.tiny_mixture(3)
    ctx.load(pb)
    # mixture mode checks its own bounds on the prune cap before anything touches the GPU
    assert code(ctx.search, se.demand_mrps, se.slo_latency_us, se.slo_accuracy, 1) in (jsv.E_BADARG, jsv.E_DEVICE)
    ctx.set_mixtures(False)


def test_static_scratch_entry_point_rejects_what_does_not_fit_before_any_device_call(ctx):
    """jsv_search_static sizes tables + workspace against JSV_STATIC_SCRATCH_BYTES on the host."""
    w = W.xr8(seed=0)
    pb, se = w.problems[0], w.searches[0]
    ctx.load(pb)
    many = np.full(2000, 50_000, dtype=np.uint32)
    assert code(ctx.search_static, many, se.slo_latency_us, se.slo_accuracy, 20) == jsv.E_WORKSPACE
    assert code(ctx.search_static, many[:0], se.slo_latency_us, se.slo_accuracy, 20) == jsv.E_BADARG
    assert code(ctx.search_static, many[:4], se.slo_latency_us, se.slo_accuracy, 3) == jsv.E_BADARG   # cap < 2V
    ctx.set_mixtures(True)
    assert code(ctx.search_static, many[:4], se.slo_latency_us, se.slo_accuracy, 20) == jsv.E_STATE
