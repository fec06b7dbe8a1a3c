"""Pins for the oracle's three convolution maps (CPU only).

None of these re-types the oracle's loops: they use a differently structured evaluator
(strided window view + einsum), library matmul for the 1x1 case, hand-worked closed forms,
adjoint identities and finite differences.
"""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

CASES = [
    # N  H  W  C  K  R  S st pad
    (2, 5, 6, 3, 4, 3, 3, 1, 1),
    (1, 7, 7, 2, 3, 3, 3, 2, 1),
    (2, 8, 6, 5, 2, 1, 1, 1, 0),
    (2, 8, 8, 3, 4, 1, 1, 2, 0),
    (1, 9, 10, 2, 3, 7, 7, 2, 3),
    (1, 6, 6, 2, 2, 3, 3, 2, 1),   # even extent, stride 2: last input row never read by r=2 at p=P-1
    (1, 5, 5, 1, 1, 5, 5, 1, 0),   # single output pixel
]


def _rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def _einsum_conv(x, w, st, pad):
    """Independent evaluator: explicit zero padding + strided window view + einsum."""
    N, H, W, C = x.shape
    K, R, S, _ = w.shape
    xp = np.zeros((N, H + 2 * pad, W + 2 * pad, C))
    xp[:, pad:pad + H, pad:pad + W, :] = x
    win = np.lib.stride_tricks.sliding_window_view(xp, (R, S), axis=(1, 2))  # N,H',W',C,R,S
    win = win[:, ::st, ::st]
    return np.einsum("npqcrs,krsc->npqk", win, w)


@pytest.mark.parametrize("case", CASES)
def test_fwd_matches_window_einsum(case):
    N, H, W, C, K, R, S, st, pad = case
    s = oracle.shape(N, H, W, C, K, R, S, st, pad)
    x, w = _rand((N, H, W, C), 1), _rand((K, R, S, C), 2)
    y = oracle.conv_fwd(s, x, w)
    ref = _einsum_conv(x, w, st, pad)
    assert y.shape == ref.shape == (N, s.P, s.Q, K)
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)


def test_fwd_1x1_is_matmul():
    N, H, W, C, K = 3, 4, 5, 7, 6
    s = oracle.shape(N, H, W, C, K, 1, 1, 1, 0)
    x, w = _rand((N, H, W, C), 3), _rand((K, 1, 1, C), 4)
    y = oracle.conv_fwd(s, x, w)
    ref = x.reshape(-1, C) @ w.reshape(K, C).T
    np.testing.assert_allclose(y.reshape(-1, K), ref, rtol=0, atol=1e-12)


def test_fwd_delta_kernel_is_shift():
    """A filter that is 1 at tap (r0,s0) for c==k copies the input shifted by (r0-pad, s0-pad)."""
    N, H, W, C = 1, 6, 7, 3
    x = _rand((N, H, W, C), 5)
    for r0 in range(3):
        for s0 in range(3):
            w = np.zeros((C, 3, 3, C))
            for c in range(C):
                w[c, r0, s0, c] = 1.0
            y = oracle.conv_fwd(oracle.shape(N, H, W, C, C, 3, 3, 1, 1), x, w)
            ref = np.zeros_like(x)
            for p in range(H):
                for q in range(W):
                    h, ww = p - 1 + r0, q - 1 + s0
                    if 0 <= h < H and 0 <= ww < W:
                        ref[0, p, q] = x[0, h, ww]
            assert np.array_equal(y, ref)


@pytest.mark.parametrize("fname,H,W,st", [("ones_3x3_pad1_6x5.txt", 6, 5, 1),
                                          ("ones_3x3_pad1_stride2_7x7.txt", 7, 7, 2)])
def test_fwd_golden_tap_counts(fname, H, W, st):
    gold = np.loadtxt(os.path.join(GOLDEN, fname))
    C = 3
    s = oracle.shape(1, H, W, C, 2, 3, 3, st, 1)
    y = oracle.conv_fwd(s, np.ones((1, H, W, C)), np.ones((2, 3, 3, C)))
    assert y.shape[1:3] == gold.shape
    for k in range(2):
        assert np.array_equal(y[0, :, :, k], gold * C)


def test_fwd_is_bilinear():
    N, H, W, C, K, R, S, st, pad = CASES[1]
    s = oracle.shape(N, H, W, C, K, R, S, st, pad)
    x1, x2 = _rand((N, H, W, C), 6), _rand((N, H, W, C), 7)
    w1, w2 = _rand((K, R, S, C), 8), _rand((K, R, S, C), 9)
    a, b = 0.7, -1.3
    np.testing.assert_allclose(oracle.conv_fwd(s, a * x1 + b * x2, w1),
                               a * oracle.conv_fwd(s, x1, w1) + b * oracle.conv_fwd(s, x2, w1), atol=1e-12)
    np.testing.assert_allclose(oracle.conv_fwd(s, x1, a * w1 + b * w2),
                               a * oracle.conv_fwd(s, x1, w1) + b * oracle.conv_fwd(s, x1, w2), atol=1e-12)


@pytest.mark.parametrize("case", CASES)
def test_adjoint_identities(case):
    """<conv(x,w), g> = <x, bwd_data(g,w)> = <w, bwd_weight(x,g)> (conv is bilinear)."""
    N, H, W, C, K, R, S, st, pad = case
    s = oracle.shape(N, H, W, C, K, R, S, st, pad)
    x, w = _rand((N, H, W, C), 10), _rand((K, R, S, C), 11)
    g = _rand((N, s.P, s.Q, K), 12)
    lhs = float(np.sum(oracle.conv_fwd(s, x, w) * g))
    dx = oracle.conv_bwd_data(s, g, w)
    dw = oracle.conv_bwd_weight(s, x, g)
    assert dx.shape == x.shape and dw.shape == w.shape
    scale = abs(lhs) + 1.0
    assert abs(lhs - float(np.sum(x * dx))) < 1e-11 * scale
    assert abs(lhs - float(np.sum(w * dw))) < 1e-11 * scale


@pytest.mark.parametrize("case", CASES[:4])
def test_gradients_match_finite_differences(case):
    """L = <conv(x,w), g> is bilinear, so central differences are exact up to round-off."""
    N, H, W, C, K, R, S, st, pad = case
    s = oracle.shape(N, H, W, C, K, R, S, st, pad)
    x, w = _rand((N, H, W, C), 13), _rand((K, R, S, C), 14)
    g = _rand((N, s.P, s.Q, K), 15)
    dx = oracle.conv_bwd_data(s, g, w)
    dw = oracle.conv_bwd_weight(s, x, g)
    rng = np.random.Generator(np.random.PCG64(16))
    eps = 0.5
    for _ in range(12):
        i = tuple(rng.integers(0, d) for d in x.shape)
        xp, xm = x.copy(), x.copy()
        xp[i] += eps
        xm[i] -= eps
        fd = (np.sum(oracle.conv_fwd(s, xp, w) * g) - np.sum(oracle.conv_fwd(s, xm, w) * g)) / (2 * eps)
        assert abs(fd - dx[i]) < 1e-10 * (1 + abs(fd))
        j = tuple(rng.integers(0, d) for d in w.shape)
        wp, wm = w.copy(), w.copy()
        wp[j] += eps
        wm[j] -= eps
        fd = (np.sum(oracle.conv_fwd(s, x, wp) * g) - np.sum(oracle.conv_fwd(s, x, wm) * g)) / (2 * eps)
        assert abs(fd - dw[j]) < 1e-10 * (1 + abs(fd))


def test_bwd_brute_force_tiny():
    """Scatter form of both gradients written from the forward definition, pure Python."""
    N, H, W, C, K, R, S, st, pad = 1, 4, 5, 2, 2, 3, 3, 2, 1
    s = oracle.shape(N, H, W, C, K, R, S, st, pad)
    x, w = _rand((N, H, W, C), 17), _rand((K, R, S, C), 18)
    g = _rand((N, s.P, s.Q, K), 19)
    dx = np.zeros_like(x)
    dw = np.zeros_like(w)
    for n in range(N):
        for p in range(s.P):
            for q in range(s.Q):
                for k in range(K):
                    for r in range(R):
                        for t in range(S):
                            h, ww = p * st - pad + r, q * st - pad + t
                            if 0 <= h < H and 0 <= ww < W:
                                for c in range(C):
                                    dx[n, h, ww, c] += g[n, p, q, k] * w[k, r, t, c]
                                    dw[k, r, t, c] += g[n, p, q, k] * x[n, h, ww, c]
    np.testing.assert_allclose(oracle.conv_bwd_data(s, g, w), dx, atol=1e-13)
    np.testing.assert_allclose(oracle.conv_bwd_weight(s, x, g), dw, atol=1e-13)


def test_bwd_data_1x1_stride2_leaves_skipped_pixels_zero():
    N, H, W, C, K = 1, 6, 6, 3, 4
    s = oracle.shape(N, H, W, C, K, 1, 1, 2, 0)
    w = _rand((K, 1, 1, C), 20)
    g = _rand((N, s.P, s.Q, K), 21)
    dx = oracle.conv_bwd_data(s, g, w)
    ref = np.zeros((N, H, W, C))
    ref[:, ::2, ::2, :] = (g.reshape(-1, K) @ w.reshape(K, C)).reshape(N, s.P, s.Q, C)
    np.testing.assert_allclose(dx, ref, atol=1e-13)


@pytest.mark.parametrize("case", CASES)
def test_sampled_evaluators_equal_full(case):
    N, H, W, C, K, R, S, st, pad = case
    s = oracle.shape(N, H, W, C, K, R, S, st, pad)
    x, w = _rand((N, H, W, C), 22), _rand((K, R, S, C), 23)
    g = _rand((N, s.P, s.Q, K), 24)
    rng = np.random.Generator(np.random.PCG64(25))
    y, dx, dw = oracle.conv_fwd(s, x, w), oracle.conv_bwd_data(s, g, w), oracle.conv_bwd_weight(s, x, g)
    for full, fn, a, b in ((y, oracle.conv_fwd_at, x, w), (dx, oracle.conv_bwd_data_at, g, w),
                           (dw, oracle.conv_bwd_weight_at, x, g)):
        idx = rng.integers(0, full.size, size=min(50, full.size))
        assert np.array_equal(fn(s, a, b, idx), full.reshape(-1)[idx])


def test_bad_shapes_are_rejected():
    s = oracle.shape(1, 4, 4, 1, 1, 3, 3, 1, 1)
    s.P = 5
    with pytest.raises(ValueError):
        oracle.conv_fwd(s, np.zeros((1, 4, 4, 1)), np.zeros((1, 3, 3, 1)))
    s = oracle.shape(1, 4, 4, 1, 1, 3, 3, 1, 1)
    with pytest.raises(ValueError):
        oracle.conv_fwd_at(s, np.zeros((1, 4, 4, 1)), np.zeros((1, 3, 3, 1)), np.array([16]))
