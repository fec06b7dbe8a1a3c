"""Pins for the oracle's layer-removal plan (CPU only)."""
import itertools

import numpy as np
import pytest

import oracle


def _rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def _block_edges(k1, k2):
    # one residual block on stream edge 0: a (0: stream -> e1), b (1: e1 -> e2), c (2: e2 -> stream)
    return [([2], [0], 6, True, True), ([0], [1], k1, False, False), ([1], [2], k2, False, False)]


def test_removed_branch_contributes_exactly_nothing():
    """y = x + c(b(a(x))) without bias: when the edge between a and b has no survivors the plan removes the whole
    branch, and the network with the branch taken out (identity) equals the network evaluated in full."""
    N, H, C0, C1, C2 = 2, 5, 6, 4, 3
    x = _rand((N, H, H, C0), 1)
    wa, wb, wc = _rand((C1, 1, 1, C0), 2), _rand((C2, 3, 3, C1), 3), _rand((C0, 1, 1, C2), 4)
    wb[:] = oracle.apply_zero(wb, zero_in=np.ones(C1, dtype=np.uint8))      # every input group of b is zero
    wa[:] = oracle.apply_zero(wa, zero_out=np.ones(C1, dtype=np.uint8))     # and every output group of a
    on_a, _ = oracle.group_norms(wa)
    _, in_b = oracle.group_norms(wb)
    keep1 = oracle.reconcile_edge([oracle.zero_groups(on_a, 1e-6)], [oracle.zero_groups(in_b, 1e-6)])
    assert int(keep1.sum()) == 0
    removed, dead, cut = oracle.plan_layer_removal(3, _block_edges(int(keep1.sum()), C2))
    assert removed == {0, 1, 2} and dead == {1, 2} and not cut
    sa, sb, sc = (oracle.shape(N, H, H, C0, C1, 1, 1, 1, 0), oracle.shape(N, H, H, C1, C2, 3, 3, 1, 1),
                  oracle.shape(N, H, H, C2, C0, 1, 1, 1, 0))
    full = x + oracle.conv_fwd(sc, oracle.conv_fwd(sb, oracle.conv_fwd(sa, x, wa), wb), wc)
    assert np.array_equal(full, x)                                           # the branch adds exact zeros
    # nothing dies while every edge keeps a survivor
    assert oracle.plan_layer_removal(3, _block_edges(1, 2)) == (set(), set(), False)


def test_propagation_shortcuts_and_cuts():
    # two blocks on one stream (edge 0): layers 0-2 and 3-5; only the first block's inner edge dies
    edges = [([2, 5], [0, 3], 8, True, True), ([0], [1], 0, False, False), ([1], [2], 5, False, False),
             ([3], [4], 7, False, False), ([4], [5], 7, False, False)]
    removed, dead, cut = oracle.plan_layer_removal(6, edges)
    assert removed == {0, 1, 2} and dead == {1, 2} and not cut
    # a plain chain image -> l0 -> l1 -> l2 -> classifier: one dead edge starves everything behind it and leaves
    # everything before it unread (the image included); the edge the classifier reads dies, so the network is cut
    chain = [([], [0], 3, True, False), ([0], [1], 4, False, False), ([1], [2], 0, False, False), ([2], [], 9, False, True)]
    removed, dead, cut = oracle.plan_layer_removal(3, chain)
    assert removed == {0, 1, 2} and dead == {0, 1, 2, 3} and cut
    # the stream itself losing every channel takes all its readers and writers along
    edges[0] = ([2, 5], [0, 3], 0, True, True)
    edges[1] = ([0], [1], 3, False, False)
    removed, dead, cut = oracle.plan_layer_removal(6, edges)
    assert removed == {0, 1, 2, 3, 4, 5} and dead == {0, 1, 2, 3, 4} and cut


def _closed(n_layers, edges, removed, dead):
    """(removed, dead) contains the seeds and is closed under the three rules."""
    for e, (prod, cons, n_keep, fed, read) in enumerate(edges):
        if n_keep == 0 and e not in dead:
            return False
        if e in dead and not (set(prod) | set(cons)) <= removed:
            return False
        if e not in dead:
            if prod and not fed and set(prod) <= removed:
                return False
            if cons and not read and set(cons) <= removed:
                return False
    return True


@pytest.mark.parametrize("seed", range(40))
def test_plan_is_the_least_closed_set_on_random_small_graphs(seed):
    rng = np.random.Generator(np.random.PCG64(seed))
    n_layers, n_edges = int(rng.integers(1, 6)), int(rng.integers(1, 5))
    edges = []
    for _ in range(n_edges):
        prod = sorted(set(rng.integers(0, n_layers, size=rng.integers(0, 3)).tolist()))
        cons = sorted(set(rng.integers(0, n_layers, size=rng.integers(0, 3)).tolist()))
        edges.append((prod, cons, int(rng.integers(0, 3)), bool(rng.integers(0, 4) == 0), bool(rng.integers(0, 4) == 0)))
    removed, dead, cut = oracle.plan_layer_removal(n_layers, edges)
    assert _closed(n_layers, edges, removed, dead)
    # brute force: the intersection of all closed sets is closed too and is the least one
    least_r, least_d = set(range(n_layers)), set(range(n_edges))
    for rbits in itertools.product([0, 1], repeat=n_layers):
        for dbits in itertools.product([0, 1], repeat=n_edges):
            r = {i for i, b in enumerate(rbits) if b}
            d = {i for i, b in enumerate(dbits) if b}
            if _closed(n_layers, edges, r, d):
                least_r &= r
                least_d &= d
    assert removed == least_r and dead == least_d
    assert cut == any(edges[e][4] for e in dead)
