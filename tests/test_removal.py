"""The library's host-only layer-removal planner against the oracle's plan (CPU only: no device work)."""
import numpy as np
import pytest

import oracle
from paper_1901_09290_amd import binding as B


def _ext(fed, read):
    return (B.EDGE_FED_OUTSIDE if fed else 0) | (B.EDGE_READ_OUTSIDE if read else 0)


@pytest.mark.parametrize("seed", range(200))
def test_planner_matches_oracle_on_random_graphs(seed):
    rng = np.random.Generator(np.random.PCG64(1000 + seed))
    n_layers, n_edges = int(rng.integers(1, 60)), int(rng.integers(1, 50))
    edges = []
    for _ in range(n_edges):
        prod = sorted(set(rng.integers(0, n_layers, size=rng.integers(0, 4)).tolist()))
        cons = sorted(set(rng.integers(0, n_layers, size=rng.integers(0, 4)).tolist()))
        edges.append((prod, cons, int(rng.integers(0, 6)), bool(rng.integers(0, 5) == 0), bool(rng.integers(0, 5) == 0)))
    removed, dead, cut = oracle.plan_layer_removal(n_layers, edges)
    got_r, got_d, rc = B.plan_layer_removal([(p, c, k, _ext(f, r)) for p, c, k, f, r in edges], n_layers)
    assert {i for i, b in enumerate(got_r) if b} == removed and {i for i, b in enumerate(got_d) if b} == dead
    assert (rc == -6) == cut


def test_planner_on_the_resnet50_graph_removes_exactly_the_starved_branches():
    from paper_1901_09290_amd import workloads as wl
    layers, edges = wl.resnet50_layers(N=1)
    n_keep = [e.n for e in edges]
    # empty the inner edge behind the first 1x1 of two bottleneck blocks
    inner = [i for i, e in enumerate(edges) if len(e.producers) == 1 and len(e.consumers) == 1]
    hit = [inner[2], inner[9]]
    for i in hit:
        n_keep[i] = 0
    desc = []
    for i, e in enumerate(edges):
        fed = len(e.producers) == 0 or len(e.producers) > 1     # image, or a residual stream (identity shortcut)
        read = len(e.consumers) == 0 or len(e.producers) > 1    # streams feed the next stage / the classifier
        desc.append((e.producers, e.consumers, n_keep[i], fed, read))
    removed, dead, cut = oracle.plan_layer_removal(len(layers), desc)
    got_r, got_d, rc = B.plan_layer_removal([(p, c, k, _ext(f, r)) for p, c, k, f, r in desc], len(layers))
    assert {i for i, b in enumerate(got_r) if b} == removed and {i for i, b in enumerate(got_d) if b} == dead
    assert rc == 0 and not cut
    assert len(removed) == 6            # two whole bottleneck branches of three convolutions each
    for i in hit:
        assert set(edges[i].producers) | set(edges[i].consumers) <= removed


def test_planner_validates_its_arguments():
    lib = B.lib()
    assert lib.pt_plan_layer_removal(None, 0, 0, None, None) == 0
    assert lib.pt_plan_layer_removal(None, 1, 1, None, None) == -1
    with pytest.raises(B.PruneTrainError) as e:
        B.plan_layer_removal([([3], [0], 1, 0)], 2)          # layer id out of range
    assert e.value.status == -2
    with pytest.raises(B.PruneTrainError) as e:
        B.plan_layer_removal([([0], [1], 1, 4)], 2)          # unknown flag bit
    assert e.value.status == -4
