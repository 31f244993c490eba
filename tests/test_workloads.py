"""The synthetic inputs: determinism, shapes, and the accuracy guard band."""
import numpy as np
import pytest

import oracle
from paper_2603_08797_amd import workloads as W


def test_splitmix64_reference_values():
    # First outputs of SplitMix64 from state 0, as published with the algorithm.
    r = W.SplitMix64()
    r.state = 0
    assert [r.next_u64() for _ in range(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4,
                                                0x06C45D188009454F]


def test_generators_are_deterministic_and_shaped():
    for name, fn in W.BENCH_WORKLOADS.items():
        a, b = fn(), fn()
        assert len(a.problems) == len(a.searches)
        for pa, pb in zip(a.problems, b.problems):
            assert np.array_equal(pa.latency_us, pb.latency_us)
            assert np.array_equal(pa.accuracy, pb.accuracy)
            assert np.array_equal(pa.src, pb.src) and np.array_equal(pa.dst, pb.dst)
            assert pa.latency_us.shape == (pa.T, pa.V, pa.P, pa.B)
            assert pa.latency_us.dtype == np.uint32 and pa.accuracy.dtype == np.float64
            assert (pa.latency_us > 0).all() and (pa.thr_mrps > 0).all()
            assert (np.diff(pa.accuracy, axis=1) >= 0).all()
    assert W.chain3().problems[0].C ** 3 == 110592
    assert W.chain4().problems[0].C ** 4 == 384160000
    assert len(W.diamond5().searches[0].demand_mrps) == 32
    d = W.xr8().searches[0].demand_mrps
    assert len(d) == 64 and d[0] == 10_000 and d[-1] == 5_000_000
    assert len(W.dagbatch().problems) == 256
    assert {p.T for p in W.dagbatch().problems} == {3, 4, 5, 6}
    t3 = W.traffic3()
    f = t3.meta["factor_milli"]
    assert f.shape == (2, 5) and f.dtype == np.uint32 and (np.diff(f.astype(np.int64), axis=1) >= 0).all()
    assert np.array_equal(f, W.traffic3().meta["factor_milli"]) and t3.problems[0].C == 245


def test_xr8_keeps_its_skeleton_and_differs_by_seed():
    for seed in range(4):
        pb = W.xr8(seed=seed).problems[0]
        edges = set(zip(pb.src.tolist(), pb.dst.tolist()))
        assert set(W.XR_SKELETON) <= edges and all(a < b for a, b in edges)
    assert not np.array_equal(W.xr8(seed=0).problems[0].latency_us,
                              W.xr8(seed=1).problems[0].latency_us)


@pytest.mark.parametrize("name,seeds", [("chain3", [0]), ("diamond5", [0]), ("chain4", [0]),
                                        ("xr8", [0, 1, 2, 3]), ("dagbatch", [0]), ("traffic3", [0])])
def test_no_candidate_within_1e_9_of_the_accuracy_slo(name, seeds):
    for seed in seeds:
        w = W.BENCH_WORKLOADS[name](seed=seed)
        for pb, se in zip(w.problems, w.searches):
            assert oracle.Oracle.from_problem(pb).accuracy_margin(se.slo_accuracy) > 1e-9


def test_sweep_crosses_from_feasible_to_infeasible():
    w = W.diamond5()
    pb, se = w.problems[0], w.searches[0]
    o = oracle.Oracle.from_problem(pb)
    ends = [int(se.demand_mrps[0]), int(se.demand_mrps[-1])]
    res, bl, md = o.search(ends, se.slo_latency_us, se.slo_accuracy, se.prune_cap, threads=8)
    assert res[0].feasible and not res[1].feasible and md == ends[0]
