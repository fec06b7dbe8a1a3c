"""Pins for the oracle's mask reconciliation, compaction plan and gathers (CPU only)."""
import itertools

import numpy as np
import pytest

import oracle
from paper_1901_09290_amd import workloads as wl


def _rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def test_reconcile_brute_force_all_masks():
    """All mask combinations for 2 producers + 1 consumer over n=3 channels (2^9 cases):
    'prune the intersection of sparsified channels' == 'keep the union of dense channels'."""
    n = 3
    for bits in itertools.product([0, 1], repeat=3 * n):
        m = np.array(bits, dtype=np.uint8).reshape(3, n)
        keep = oracle.reconcile_edge([m[0], m[1]], [m[2]])
        dense_union = (1 - m[0]) | (1 - m[1]) | (1 - m[2])     # union of dense sets
        sparse_inter = m[0] & m[1] & m[2]                        # intersection of sparsified sets
        assert np.array_equal(keep, dense_union)
        assert np.array_equal(keep, 1 - sparse_inter)


def test_reconcile_pair_and_union_superset():
    rng = np.random.Generator(np.random.PCG64(1))
    masks = [(rng.random(40) < 0.5).astype(np.uint8) for _ in range(7)]
    keep = oracle.reconcile_edge(masks[:3], masks[3:])
    for m in masks:
        assert np.all(keep >= (1 - m))          # union contains every member's dense set
    # adjacent pair: one producer, one consumer
    k2 = oracle.reconcile_edge([masks[0]], [masks[1]])
    assert np.array_equal(k2, 1 - (masks[0] & masks[1]))
    # producers only (a node whose readers are outside the conv set)
    k3 = oracle.reconcile_edge([masks[0], masks[1]], [])
    assert np.array_equal(k3, 1 - (masks[0] & masks[1]))


def test_plan_properties_all_masks_up_to_8():
    for n in range(0, 9):
        for bits in itertools.product([0, 1], repeat=n):
            keep = np.array(bits, dtype=np.uint8)
            idx = oracle.compact_plan(keep)
            assert idx.size == int(keep.sum())
            assert np.all(np.diff(idx) > 0)
            assert np.all(keep[idx] == 1) if idx.size else True
            assert idx.tolist() == [j for j in range(n) if bits[j]]


def test_gathers_match_numpy_indexing():
    w = _rand((7, 3, 3, 9), 2)
    ik = np.array([0, 2, 3, 6], dtype=np.int32)
    ic = np.array([1, 4, 5, 7, 8], dtype=np.int32)
    assert np.array_equal(oracle.compact_weights(w, ik, ic), w[ik][..., ic])
    assert np.array_equal(oracle.compact_weights(w, None, ic), w[..., ic])
    assert np.array_equal(oracle.compact_weights(w, ik, None), w[ik])
    v = _rand((7,), 3).astype(np.float32)
    assert np.array_equal(oracle.compact_vector(v, ik), v[ik])
    x = (_rand((2, 4, 5, 9), 4) * 100).astype(np.int16)       # 2-byte elements, like bf16 bits
    assert np.array_equal(oracle.compact_nhwc(x, ic), x[..., ic])
    # scatter(gather(v)) restores a tensor whose dropped entries are zero
    vz = v.copy()
    drop = np.setdiff1d(np.arange(7), ik)
    vz[drop] = 0
    back = np.zeros_like(vz)
    back[ik] = oracle.compact_vector(vz, ik)
    assert np.array_equal(back, vz)


@pytest.mark.parametrize("st,R,pad", [(1, 3, 1), (2, 3, 1), (1, 1, 0), (2, 1, 0)])
def test_compacted_layer_computes_the_same_function(st, R, pad):
    """A layer whose zero groups are removed gives bit-identical results on the kept channels and
    exact zeros on the dropped ones: the dropped terms are exact +0 products and the loop order
    over survivors is unchanged."""
    N, H, W, C, K = 2, 8, 8, 10, 12
    rng = np.random.Generator(np.random.PCG64(5))
    x = _rand((N, H, W, C), 6)
    w = _rand((K, R, R, C), 7)
    zi = np.sort(rng.choice(C, 3, replace=False))
    zo = np.sort(rng.choice(K, 4, replace=False))
    w = wl.zero_groups_in_weights(w, zo, zi)
    s = oracle.shape(N, H, W, C, K, R, R, st, pad)
    on, inn = oracle.group_norms(w)
    keep_k = 1 - oracle.zero_groups(on, 1e-6)
    keep_c = 1 - oracle.zero_groups(inn, 1e-6)
    ik, ic = oracle.compact_plan(keep_k), oracle.compact_plan(keep_c)
    assert ik.tolist() == np.setdiff1d(np.arange(K), zo).tolist()
    assert ic.tolist() == np.setdiff1d(np.arange(C), zi).tolist()
    wc = oracle.compact_weights(w, ik, ic)
    xc = oracle.compact_nhwc(x, ic)
    sc = oracle.shape(N, H, W, ic.size, ik.size, R, R, st, pad)

    y = oracle.conv_fwd(s, x, w)
    yc = oracle.conv_fwd(sc, xc, wc)
    assert np.array_equal(y[..., ik], yc)
    assert np.all(y[..., zo] == 0.0)

    g = _rand(y.shape, 8)
    gc = oracle.compact_nhwc(g, ik)
    dx = oracle.conv_bwd_data(s, g, w)
    dxc = oracle.conv_bwd_data(sc, gc, wc)
    assert np.array_equal(dx[..., ic], dxc)
    assert np.all(dx[..., zi] == 0.0)

    dw = oracle.conv_bwd_weight(s, x, g)
    dwc = oracle.conv_bwd_weight(sc, xc, gc)
    assert np.array_equal(oracle.compact_weights(dw, ik, ic), dwc)


def test_residual_stage_channel_union_preserves_function():
    """Two basic blocks sharing one node (ReLU + add glue): zero a channel set consistently on the
    node (producers' out-groups and consumers' in-groups) and on the block-internal edges, derive
    keep masks through norms -> zero_groups -> reconcile -> plan, compact everything, and check that
    the compacted stack equals the original stack on the kept node channels."""
    N, H, Cn, Cm = 2, 6, 8, 6
    rng = np.random.Generator(np.random.PCG64(9))
    x = np.maximum(_rand((N, H, H, Cn), 10), 0)
    # convs: a1: node->m1, b1: m1->node, a2: node->m2, b2: m2->node
    wa1, wb1 = _rand((Cm, 3, 3, Cn), 11), _rand((Cn, 3, 3, Cm), 12)
    wa2, wb2 = _rand((Cm, 3, 3, Cn), 13), _rand((Cn, 3, 3, Cm), 14)
    zn = np.sort(rng.choice(Cn, 3, replace=False))
    z1 = np.sort(rng.choice(Cm, 2, replace=False))
    z2 = np.sort(rng.choice(Cm, 1, replace=False))
    wa1 = wl.zero_groups_in_weights(wa1, z1, zn)
    wb1 = wl.zero_groups_in_weights(wb1, zn, z1)
    wa2 = wl.zero_groups_in_weights(wa2, z2, zn)
    wb2 = wl.zero_groups_in_weights(wb2, zn, z2)
    # make one node channel zero in only SOME members: it must survive (union of dense channels)
    extra = int(np.setdiff1d(np.arange(Cn), zn)[0])
    wb1[extra] = 0.0
    x[..., zn] = 0.0   # the node's incoming feature has nothing on channels nobody writes or reads

    def stack(x, wa1, wb1, wa2, wb2):
        cn, cm1, cm2 = x.shape[-1], wa1.shape[0], wa2.shape[0]
        t = np.maximum(oracle.conv_fwd(oracle.shape(N, H, H, cn, cm1, 3, 3, 1, 1), x, wa1), 0)
        x1 = np.maximum(x + oracle.conv_fwd(oracle.shape(N, H, H, cm1, cn, 3, 3, 1, 1), t, wb1), 0)
        t = np.maximum(oracle.conv_fwd(oracle.shape(N, H, H, cn, cm2, 3, 3, 1, 1), x1, wa2), 0)
        return np.maximum(x1 + oracle.conv_fwd(oracle.shape(N, H, H, cm2, cn, 3, 3, 1, 1), t, wb2), 0)

    def zeros(w, thr=1e-6):
        on, inn = oracle.group_norms(w)
        return oracle.zero_groups(on, thr), oracle.zero_groups(inn, thr)

    (za1o, za1i), (zb1o, zb1i), (za2o, za2i), (zb2o, zb2i) = zeros(wa1), zeros(wb1), zeros(wa2), zeros(wb2)
    keep_n = oracle.reconcile_edge([zb1o, zb2o], [za1i, za2i])
    keep_1 = oracle.reconcile_edge([za1o], [zb1i])
    keep_2 = oracle.reconcile_edge([za2o], [zb2i])
    i_n, i_1, i_2 = oracle.compact_plan(keep_n), oracle.compact_plan(keep_1), oracle.compact_plan(keep_2)
    assert i_n.tolist() == np.setdiff1d(np.arange(Cn), zn).tolist() and extra in i_n
    assert i_1.tolist() == np.setdiff1d(np.arange(Cm), z1).tolist()
    assert i_2.tolist() == np.setdiff1d(np.arange(Cm), z2).tolist()

    full = stack(x, wa1, wb1, wa2, wb2)
    small = stack(oracle.compact_nhwc(x, i_n),
                  oracle.compact_weights(wa1, i_1, i_n), oracle.compact_weights(wb1, i_n, i_1),
                  oracle.compact_weights(wa2, i_2, i_n), oracle.compact_weights(wb2, i_n, i_2))
    assert np.array_equal(full[..., i_n], small)
    assert np.all(full[..., zn] == 0.0)


def test_workload_tables():
    """Layer tables: counts, parameter totals and FLOPs of the two networks."""
    l50, e50 = wl.resnet50_layers()
    assert len(l50) == 53 and len(e50) == 37
    assert sum(l.params for l in l50) == 23_454_912
    assert len(wl.distinct_shapes(l50)) == 23
    assert abs(sum(l.flops for l in l50) / 1e9 - 523.2) < 0.5
    l32, e32 = wl.resnet32_layers()
    assert len(l32) == 33 and len(e32) == 18
    assert sum(l.params for l in l32) == 463_792
    for layers, edges in ((l50, e50), (l32, e32)):
        for e in edges:
            assert all(layers[i].K == e.n for i in e.producers)
            assert all(layers[i].C == e.n for i in e.consumers)
            assert len(e.producers) >= 1
    keep = wl.pruned_keep_sets(e50, seed=3)
    assert all(k.size % 16 != 0 and 1 <= k.size <= e.n for k, e in zip(keep, e50))
    lp, ep = wl.with_widths(l50, e50, [k.size for k in keep])
    assert lp[0].C == 3 and all(l.C == ep[l.in_edge].n for l in lp if l.in_edge is not None)


# ---- channel scatter, max-abs criterion, writing flagged groups to zero --------------------------------- #
def test_scatter_is_the_inverse_of_gather_on_kept_channels():
    rng = np.random.Generator(np.random.PCG64(301))
    for C, pixels in ((5, 7), (16, 33), (37, 10)):
        x = rng.integers(1, 60000, size=(pixels, C)).astype(np.uint16)        # no zeros in the data
        idx = np.sort(rng.choice(C, max(1, C * 2 // 3), replace=False)).astype(np.int32)
        g = oracle.compact_nhwc(x, idx)
        s = oracle.scatter_nhwc(g, idx, C)
        want = np.zeros_like(x)
        want[:, idx] = x[:, idx]                                             # numpy fancy indexing as the second evaluator
        assert np.array_equal(s, want)
        assert np.array_equal(oracle.compact_nhwc(s, idx), g)                # gather is a left inverse of scatter
        dropped = np.setdiff1d(np.arange(C), idx)
        assert not s[:, dropped].any()
    # hand-worked: 1 pixel, Cp = 2 survivors at positions 1 and 3 of C = 4
    assert oracle.scatter_nhwc(np.array([[7, 9]], dtype=np.uint16), [1, 3], 4).tolist() == [[0, 7, 0, 9]]
    with pytest.raises(Exception):
        oracle.scatter_nhwc(np.array([[7, 9]], dtype=np.uint16), [3, 1], 4)   # not ascending


def test_group_maxabs_matches_numpy_and_bounds_the_l2_norm():
    rng = np.random.Generator(np.random.PCG64(302))
    w = rng.standard_normal((6, 3, 3, 5))
    w[2] = 0.0
    w[..., 4] = 0.0
    om, im = oracle.group_maxabs(w)
    assert np.array_equal(om, np.abs(w).max(axis=(1, 2, 3))) and np.array_equal(im, np.abs(w).max(axis=(0, 1, 2)))
    on, inn = oracle.group_norms(w)
    # max|g| <= ||g||_2 <= sqrt(size) * max|g|: the L2 criterion never flags a group the max-abs one would keep
    assert np.all(om <= on + 1e-15) and np.all(on <= np.sqrt(45) * om + 1e-12)
    assert np.all(im <= inn + 1e-15) and np.all(inn <= np.sqrt(54) * im + 1e-12)
    assert om[2] == 0.0 and im[4] == 0.0
    # both criteria agree on exactly-zero groups, whatever the threshold
    for thr in (1e-6, 1e-4):
        assert np.array_equal(oracle.zero_groups(om, thr) & (on == 0), oracle.zero_groups(on, thr) & (on == 0))
    # hand-worked 2x1x1x2 example of the golden file: w = [[3, 0], [4, 0]]
    om, im = oracle.group_maxabs(np.array([[3.0, 0.0], [-4.0, 0.0]]).reshape(2, 1, 1, 2))
    assert om.tolist() == [3.0, 4.0] and im.tolist() == [4.0, 0.0]


def test_apply_zero_writes_exact_zeros_and_makes_the_groups_detectable():
    rng = np.random.Generator(np.random.PCG64(303))
    w = rng.standard_normal((5, 2, 2, 4)) * 1e-5 + 1.0
    zo = np.array([0, 1, 0, 0, 1], dtype=np.uint8)
    zi = np.array([1, 0, 0, 0], dtype=np.uint8)
    z = oracle.apply_zero(w, zo, zi)
    want = w.copy()
    want[zo.astype(bool)] = 0.0
    want[..., zi.astype(bool)] = 0.0
    assert np.array_equal(z, want)
    assert np.array_equal(oracle.apply_zero(w, None, zi), np.where(zi.astype(bool), 0.0, w))
    assert np.array_equal(oracle.apply_zero(w, None, None), w)
    on, inn = oracle.group_norms(z)
    assert np.array_equal(oracle.zero_groups(on, 1e-6), zo) and np.array_equal(oracle.zero_groups(inn, 1e-6), zi)
    assert np.array_equal(oracle.apply_zero(z, zo, zi), z)                      # idempotent
