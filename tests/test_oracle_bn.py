"""Pins for the oracle's feature normalisation (CPU only)."""
import numpy as np

import oracle


def _rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def test_forward_matches_numpy_statistics_and_normalises():
    x = _rand((3, 5, 4, 6), 1) * 2.5 + 0.7
    gamma, beta = _rand(6, 2), _rand(6, 3)
    y, mean, invstd = oracle.bn_fwd(x, gamma, beta, 1e-5)
    flat = x.reshape(-1, 6)
    np.testing.assert_allclose(mean, flat.mean(axis=0), rtol=1e-13)
    np.testing.assert_allclose(invstd, 1.0 / np.sqrt(flat.var(axis=0) + 1e-5), rtol=1e-13)   # numpy's var is the biased one
    # with gamma = 1, beta = 0 and eps = 0 every channel of the output has mean 0 and variance 1
    y1, _, _ = oracle.bn_fwd(x, np.ones(6), np.zeros(6), 0.0)
    np.testing.assert_allclose(y1.reshape(-1, 6).mean(axis=0), 0.0, atol=1e-13)
    np.testing.assert_allclose(y1.reshape(-1, 6).var(axis=0), 1.0, rtol=1e-12)
    np.testing.assert_allclose(y, (x - flat.mean(axis=0)) / np.sqrt(flat.var(axis=0) + 1e-5) * gamma + beta, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(y, y1 * gamma + beta, atol=2e-5)                    # eps = 1e-5 vs 0 moves y by ~eps/(2 var)
    # hand-worked: channel values {1, 3}: mean 2, biased var 1 -> normalised {-1, +1}; gamma 2, beta 10 -> {8, 12}
    y2, m2, s2 = oracle.bn_fwd(np.array([[1.0], [3.0]]), [2.0], [10.0], 0.0)
    assert m2.tolist() == [2.0] and s2.tolist() == [1.0] and y2.reshape(-1).tolist() == [8.0, 12.0]
    # invariance: shifting and positively scaling a channel's input does not change the output (eps = 0)
    y3, _, _ = oracle.bn_fwd(x * 3.0 + 11.0, gamma, beta, 0.0)
    y0, _, _ = oracle.bn_fwd(x, gamma, beta, 0.0)
    np.testing.assert_allclose(y3, y0, rtol=1e-10, atol=1e-10)


def test_backward_matches_finite_differences_of_the_forward():
    x = _rand((2, 3, 3, 4), 5)
    gamma, beta = _rand(4, 6) + 1.5, _rand(4, 7)
    g = _rand((2, 3, 3, 4), 8)                      # upstream gradient: L = <y, g>
    eps = 1e-3
    _, mean, invstd = oracle.bn_fwd(x, gamma, beta, eps)
    dx, dgamma, dbeta = oracle.bn_bwd(x, g, gamma, mean, invstd)

    def loss(xx, gg, bb):
        return float(np.sum(oracle.bn_fwd(xx, gg, bb, eps)[0] * g))

    rng = np.random.Generator(np.random.PCG64(9))
    h = 1e-6
    for _ in range(20):
        i = tuple(rng.integers(0, d) for d in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        assert abs((loss(xp, gamma, beta) - loss(xm, gamma, beta)) / (2 * h) - dx[i]) < 1e-7
    for c in range(4):
        e = np.zeros(4)
        e[c] = h
        assert abs((loss(x, gamma + e, beta) - loss(x, gamma - e, beta)) / (2 * h) - dgamma[c]) < 1e-7
        assert abs((loss(x, gamma, beta + e) - loss(x, gamma, beta - e)) / (2 * h) - dbeta[c]) < 1e-7


def test_backward_identities():
    x = _rand((4, 2, 2, 3), 11)
    gamma, beta = _rand(3, 12) + 2.0, _rand(3, 13)
    g = _rand((4, 2, 2, 3), 14)
    _, mean, invstd = oracle.bn_fwd(x, gamma, beta, 1e-5)
    dx, dgamma, dbeta = oracle.bn_bwd(x, g, gamma, mean, invstd)
    np.testing.assert_allclose(dbeta, g.reshape(-1, 3).sum(axis=0), rtol=1e-13)
    # the output is invariant to a per-channel shift of x, so dx sums to zero over the batch in every channel
    np.testing.assert_allclose(dx.reshape(-1, 3).sum(axis=0), 0.0, atol=1e-12)
    # ... and (eps -> 0) to a per-channel scaling, so <dx, x - mean> vanishes up to the eps term
    xh = (x - mean) * invstd
    assert np.all(np.abs((dx * xh).reshape(-1, 3).sum(axis=0)) < 1e-3)
    # a compacted tensor gives the kept channels' results exactly (per-channel independence)
    keep = [0, 2]
    dx2, dg2, db2 = oracle.bn_bwd(x[..., keep], g[..., keep], gamma[keep], mean[keep], invstd[keep])
    assert np.array_equal(dx2, dx[..., keep]) and np.array_equal(dg2, dgamma[keep]) and np.array_equal(db2, dbeta[keep])
