"""Graph mode: the recorded launch sequence must give, on every replay, what the eager
sequence gives - with other work and synchronisations in between, with new demands
travelling through the same graph, and across shape changes that force a new recording."""
import numpy as np
import pytest

from paper_2603_08797_amd import jsv, workloads as W

pytestmark = pytest.mark.gpu


def strip(res):
    return [(r.feasible, r.index, r.cost, r.latency_us, r.choice, r.replicas, r.evaluated, r.flags, r.accuracy)
            for r in res]


def test_replays_match_eager_runs():
    import torch
    eager, graph = jsv.Jsv(device=0), jsv.Jsv(device=0, stream=torch.cuda.Stream())
    graph.set_graph_mode(True)
    w = W.diamond5()
    pb, se = w.problems[0], w.searches[0]
    eager.load(pb)
    graph.load(pb)
    rng = np.random.default_rng(3)
    junk = torch.zeros(1 << 20, device="cuda")
    for rep in range(6):
        dem = np.sort(rng.integers(5_000, 900_000, size=len(se.demand_mrps))).astype(np.uint32)
        slo_l = int(rng.integers(60_000, 140_000))
        a, sa = eager.search(dem, slo_l, se.slo_accuracy, se.prune_cap)
        junk += 1.0                                  # unrelated eager work between replays
        torch.cuda.synchronize()
        b, sb = graph.search(dem, slo_l, se.slo_accuracy, se.prune_cap)
        assert strip(a) == strip(b), f"replay {rep}"
        assert (sa.best_level, sa.max_demand_mrps) == (sb.best_level, sb.max_demand_mrps)
        assert sb.seconds_device > 0 and sb.seconds_enumerate == 0
    # another shape (fewer levels, other cap) records again; then the first shape once more
    a, _ = eager.search(se.demand_mrps[:5], se.slo_latency_us, se.slo_accuracy, 0)
    b, _ = graph.search(se.demand_mrps[:5], se.slo_latency_us, se.slo_accuracy, 0)
    assert strip(a) == strip(b)
    a, _ = eager.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    b, _ = graph.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    assert strip(a) == strip(b)
    # objective mode is part of the recorded shape
    for j in (eager, graph):
        j.set_objective(1, 1.0, 0.035)
    a, _ = eager.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    b, _ = graph.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    assert strip(a) == strip(b) and [r.objective for r in a] == [r.objective for r in b]
    graph.set_graph_mode(False)                      # back to eager launches on the same context
    graph.set_objective(0)
    eager.set_objective(0)
    a, _ = eager.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    b, sb = graph.search(se.demand_mrps, se.slo_latency_us, se.slo_accuracy, se.prune_cap)
    assert strip(a) == strip(b) and sb.seconds_enumerate > 0
    eager.close()
    graph.close()


def test_batch_replays():
    import torch
    w = W.dagbatch(n=32)
    eager, graph = jsv.Jsv(device=0), jsv.Jsv(device=0, stream=torch.cuda.Stream())
    with pytest.raises(jsv.JsvError) as e:           # the default stream cannot be captured
        eager.set_graph_mode(True)
    assert e.value.code == jsv.E_STATE
    graph.set_graph_mode(True)
    eager.load_batch(w.problems, w.searches)
    graph.load_batch(w.problems, w.searches)
    a, _ = eager.search_loaded_batch()
    for _ in range(4):
        b, _ = graph.search_loaded_batch()
        assert strip(a) == strip(b)
    eager.close()
    graph.close()
