"""Pins for the oracle's group norms, group-lasso gradient and zero-group detection (CPU only)."""
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand(shape, seed):
    return np.random.Generator(np.random.PCG64(seed)).standard_normal(shape)


def _golden():
    out = {}
    with open(os.path.join(GOLDEN, "group_lasso_2x1x2.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            k, *v = line.split()
            out[k] = np.array([float(t) for t in v])
    return out


def test_golden_hand_example():
    g = _golden()
    w = np.array([[3.0, 0.0], [4.0, 0.0]]).reshape(2, 1, 1, 2)
    on, inn = oracle.group_norms(w)
    assert np.array_equal(on, g["out_norm"]) and np.array_equal(inn, g["in_norm"])
    assert on.sum() + inn.sum() == g["penalty"][0]
    grad = oracle.group_lasso_grad(w, on, inn, 0.5, 3, np.zeros_like(w))
    np.testing.assert_allclose(grad.reshape(-1), g["grad"], rtol=0, atol=1e-15)


@pytest.mark.parametrize("shape", [(5, 3, 3, 7), (8, 1, 1, 3), (3, 7, 7, 2)])
def test_norms_match_numpy_linalg(shape):
    w = _rand(shape, 1)
    on, inn = oracle.group_norms(w)
    K, C = shape[0], shape[-1]
    np.testing.assert_allclose(on, np.linalg.norm(w.reshape(K, -1), axis=1), rtol=1e-14)
    np.testing.assert_allclose(inn, np.linalg.norm(w.reshape(-1, C), axis=0), rtol=1e-14)
    # every weight sits in exactly one group of each kind
    fro2 = float(np.sum(w * w))
    assert abs(np.sum(on ** 2) - fro2) < 1e-12 * fro2
    assert abs(np.sum(inn ** 2) - fro2) < 1e-12 * fro2


def test_grad_closed_form_per_group():
    w = _rand((6, 3, 3, 5), 2)
    on, inn = oracle.group_norms(w)
    lam = 0.37
    z = np.zeros_like(w)
    g_out = oracle.group_lasso_grad(w, on, inn, lam, 1, z)
    g_in = oracle.group_lasso_grad(w, on, inn, lam, 2, z)
    g_both = oracle.group_lasso_grad(w, on, inn, lam, 3, z)
    for k in range(6):
        np.testing.assert_allclose(g_out[k], lam * w[k] / np.linalg.norm(w[k]), rtol=1e-13)
        # with only output groups, each filter's gradient has L2 norm exactly lambda
        assert abs(np.linalg.norm(g_out[k]) - lam) < 1e-13
    for c in range(5):
        np.testing.assert_allclose(g_in[..., c], lam * w[..., c] / np.linalg.norm(w[..., c]), rtol=1e-13)
    np.testing.assert_allclose(g_both, g_out + g_in, rtol=1e-13)
    assert np.array_equal(oracle.group_lasso_grad(w, on, inn, lam, 0, z), z)


def test_grad_accumulates_onto_dw():
    w = _rand((4, 1, 1, 3), 3)
    dw0 = _rand((4, 1, 1, 3), 4)
    on, inn = oracle.group_norms(w)
    g = oracle.group_lasso_grad(w, on, inn, 0.1, 3, np.zeros_like(w))
    np.testing.assert_allclose(oracle.group_lasso_grad(w, on, inn, 0.1, 3, dw0), dw0 + g, rtol=1e-14)


def test_grad_matches_finite_differences_of_penalty():
    w = _rand((4, 3, 3, 3), 5)
    lam = 1e-2

    def penalty(v):
        on, inn = oracle.group_norms(v)
        return lam * (on.sum() + inn.sum())

    on, inn = oracle.group_norms(w)
    g = oracle.group_lasso_grad(w, on, inn, lam, 3, np.zeros_like(w))
    rng = np.random.Generator(np.random.PCG64(6))
    eps = 1e-6
    for _ in range(25):
        i = tuple(rng.integers(0, d) for d in w.shape)
        wp, wm = w.copy(), w.copy()
        wp[i] += eps
        wm[i] -= eps
        fd = (penalty(wp) - penalty(wm)) / (2 * eps)
        assert abs(fd - g[i]) < 1e-8


def test_euler_identity_and_scale_invariance():
    w = _rand((5, 3, 3, 4), 7)
    lam = 0.2
    on, inn = oracle.group_norms(w)
    g = oracle.group_lasso_grad(w, on, inn, lam, 3, np.zeros_like(w))
    # penalty is homogeneous of degree 1: <w, grad> = lambda * penalty
    assert abs(np.sum(w * g) - lam * (on.sum() + inn.sum())) < 1e-12
    on2, in2 = oracle.group_norms(3.5 * w)
    np.testing.assert_allclose(on2, 3.5 * on, rtol=1e-14)
    g2 = oracle.group_lasso_grad(3.5 * w, on2, in2, lam, 3, np.zeros_like(w))
    np.testing.assert_allclose(g2, g, rtol=1e-13)


def test_zero_groups_get_zero_gradient_and_are_detected():
    w = _rand((6, 3, 3, 5), 8)
    w[2] = 0.0
    w[..., 4] = 0.0
    on, inn = oracle.group_norms(w)
    assert on[2] == 0.0 and inn[4] == 0.0
    g = oracle.group_lasso_grad(w, on, inn, 1.0, 3, np.zeros_like(w))
    assert np.all(g[2] == 0.0) and np.all(g[..., 4] == 0.0)
    assert np.all(np.isfinite(g))
    zo, zi = oracle.zero_groups(on, 1e-6), oracle.zero_groups(inn, 1e-6)
    assert zo.tolist() == [0, 0, 1, 0, 0, 0] and zi.tolist() == [0, 0, 0, 0, 1]


def test_zero_groups_threshold_is_strict():
    n = np.array([0.0, 1e-4, 0.99e-4, 1.01e-4, 5.0])
    assert oracle.zero_groups(n, 1e-4).tolist() == [1, 0, 1, 0, 0]
    assert oracle.zero_groups(n, 0.0).tolist() == [0, 0, 0, 0, 0]
    assert oracle.zero_groups(n, -1.0).tolist() == [0, 0, 0, 0, 0]
    # L2 norm is never below the largest magnitude in the group, so a norm test prunes no more
    # than the paper's max-abs wording (Sec. 4.2) and both agree on exactly-zero groups
    w = _rand((4, 3, 3, 4), 9) * 1e-4
    on, _ = oracle.group_norms(w)
    assert np.all(on >= np.abs(w).reshape(4, -1).max(axis=1))


def test_penalty_value_and_first_layer_exemption():
    """GroupLassoReg of Alg. 1: the plain sum of group norms, one global coefficient (no size weighting);
    flags drop a layer's input or output groups.  Pinned to the hand example and to numpy sums."""
    g = _golden()
    w = np.array([[3.0, 0.0], [4.0, 0.0]]).reshape(2, 1, 1, 2)
    on, inn = oracle.group_norms(w)
    assert oracle.group_lasso_penalty([(on, inn, 3)]) == g["penalty"][0]
    assert oracle.group_lasso_penalty([(on, inn, 1)]) == g["penalty_out_only"][0]
    assert oracle.group_lasso_penalty([(on, inn, 0)]) == 0.0
    layers, want = [], 0.0
    for i, shape in enumerate([(8, 3, 3, 3), (16, 1, 1, 8), (5, 3, 3, 16)]):
        v = _rand(shape, 40 + i)
        a, b = oracle.group_norms(v)
        flags = 1 if i == 0 else 3          # the first convolution's input groups are exempt
        layers.append((a, b, flags))
        want += np.sqrt((v ** 2).sum(axis=(1, 2, 3))).sum()
        if flags & 2:
            want += np.sqrt((v ** 2).sum(axis=(0, 1, 2))).sum()
    assert abs(oracle.group_lasso_penalty(layers) - want) < 1e-12 * want


def test_penalty_is_what_the_gradient_differentiates():
    """Finite differences of the oracle's own penalty value (not a retyped formula) reproduce the oracle's gradient,
    including the exemption flags."""
    w = _rand((4, 3, 3, 3), 55)
    for flags in (1, 2, 3):
        on, inn = oracle.group_norms(w)
        g = oracle.group_lasso_grad(w, on, inn, 1.0, flags, np.zeros_like(w))
        rng = np.random.Generator(np.random.PCG64(56))
        for _ in range(10):
            i = tuple(rng.integers(0, d) for d in w.shape)
            wp, wm = w.copy(), w.copy()
            wp[i] += 1e-6
            wm[i] -= 1e-6
            pp = oracle.group_lasso_penalty([(*oracle.group_norms(wp), flags)])
            pm = oracle.group_lasso_penalty([(*oracle.group_norms(wm), flags)])
            assert abs((pp - pm) / 2e-6 - g[i]) < 1e-8


def test_set_coeff_solves_the_penalty_ratio_equation():
    g = _golden()
    lam = oracle.set_coeff(g["set_coeff_loss1"][0], g["penalty"][0], g["set_coeff_ratio"][0])
    assert lam == g["set_coeff_lambda"][0]
    rng = np.random.Generator(np.random.PCG64(57))
    for _ in range(20):
        l1, l2, r = rng.uniform(0.1, 10), rng.uniform(1, 5000), rng.uniform(0.05, 0.6)
        lam = oracle.set_coeff(l1, l2, r)
        assert abs(lam * l2 / (l1 + lam * l2) - r) < 1e-14      # plugging back gives the wanted ratio
    # larger wanted ratio -> larger coefficient; invalid inputs are refused
    assert oracle.set_coeff(2.0, 100.0, 0.25) > oracle.set_coeff(2.0, 100.0, 0.20)
    for bad in ((1.0, 10.0, 0.0), (1.0, 10.0, 1.0), (1.0, 0.0, 0.2), (-1.0, 10.0, 0.2)):
        with pytest.raises(Exception):
            oracle.set_coeff(*bad)


def test_optimizer_step_reduces_to_known_rules():
    """SGD-with-momentum step with the regulariser folded in: special cases with textbook closed forms."""
    w, dw, m = _rand((4, 3, 3, 5), 70), _rand((4, 3, 3, 5), 71), _rand((4, 3, 3, 5), 72)
    on, inn = oracle.group_norms(w)
    # no momentum, no decay, no regulariser: plain gradient descent
    w2, m2 = oracle.sgd_momentum_lasso(w, dw, m, on, inn, 0.0, 0.1, 0.0, 0.0, 3)
    np.testing.assert_allclose(w2, w - 0.1 * dw, rtol=0, atol=1e-15)
    np.testing.assert_array_equal(m2, dw)
    # the regulariser's part equals the separately pinned lasso gradient; the rest is v = mu*v + g, w -= lr*v
    lam, lr, mu, wd = 1e-2, 0.05, 0.9, 1e-4
    g = oracle.group_lasso_grad(w, on, inn, lam, 3, dw) + wd * w
    w2, m2 = oracle.sgd_momentum_lasso(w, dw, m, on, inn, lam, lr, mu, wd, 3)
    np.testing.assert_allclose(m2, mu * m + g, rtol=1e-14)
    np.testing.assert_allclose(w2, w - lr * (mu * m + g), rtol=1e-14, atol=1e-15)
    # constant gradient, zero start: after n steps the velocity is g*(1 - mu^n)/(1 - mu) (geometric series)
    wc, mc = np.zeros((2, 1, 1, 2)), np.zeros((2, 1, 1, 2))
    gc = np.full((2, 1, 1, 2), 2.0)
    ones = np.ones(2)
    for n in range(1, 6):
        wc, mc = oracle.sgd_momentum_lasso(wc, gc, mc, ones, ones, 0.0, 0.1, 0.5, 0.0, 0)
        np.testing.assert_allclose(mc, 2.0 * (1 - 0.5 ** n) / 0.5, rtol=1e-14)


def test_optimizer_step_keeps_zeroed_groups_zero_and_descends_the_regularised_loss():
    w = _rand((6, 2, 2, 4), 73)
    w[1] = 0.0
    w[..., 2] = 0.0
    on, inn = oracle.group_norms(w)
    dw = _rand((6, 2, 2, 4), 74)
    dw[1] = 0.0            # a zeroed filter receives no loss gradient through a zero weight path in these tests
    dw[..., 2] = 0.0
    m = np.zeros_like(w)
    w2, m2 = oracle.sgd_momentum_lasso(w, dw, m, on, inn, 0.1, 0.1, 0.9, 1e-4, 3)
    assert not w2[1].any() and not w2[..., 2].any() and not m2[1].any()        # zero sub-gradient at zero groups
    # with dw = 0 a small step decreases the penalty (descent direction of lambda * sum of norms)
    pen = lambda v: oracle.group_lasso_penalty([(*oracle.group_norms(v), 3)])
    w3, _ = oracle.sgd_momentum_lasso(w, np.zeros_like(w), m, on, inn, 0.1, 1e-3, 0.0, 0.0, 3)
    assert pen(w3) < pen(w)
