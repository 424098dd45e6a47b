"""Pins of the oracle's gate activation (paper Sec. 3.2, the definition of alpha from h and beta;
Alg. 1, the overflow-safe softplus; Sec. 3.3, epsilon in the denominator) and of its derivative.

None of these checks re-types the oracle's formula: they use closed forms, the textbook
log1p(exp(z)) where it is safe, limits, monotonicity and finite differences.
"""
import numpy as np
import pytest


def test_closed_forms(oracle):
    # beta = 1, eps = 0: alpha = softplus(h); softplus(0) = ln 2
    a = oracle.gate_activation(np.array([0.0]), np.array([1.0]), 0.0)
    assert abs(a[0] - np.log(2.0)) < 1e-15
    # softplus(z) - softplus(-z) = z for every z
    h = np.linspace(-30, 30, 121)
    ap = oracle.gate_activation(h, np.ones_like(h), 0.0)
    am = oracle.gate_activation(-h, np.ones_like(h), 0.0)
    np.testing.assert_allclose(ap - am, h, rtol=0, atol=1e-12)


def test_matches_textbook_softplus_where_that_is_safe(oracle):
    rng = np.random.default_rng(1)
    h = rng.normal(size=2000) * 3
    beta = 1.0 + rng.uniform(-0.9, 3.0, size=2000)   # 1 + elu(.) lies in (0, inf)
    eps = 1e-6
    ref = np.log1p(np.exp(beta * h)) / (beta + eps)
    # the form of Alg. 1 adds 1 to exp(z) before the log: absolute, not relative, accuracy for z << 0
    np.testing.assert_allclose(oracle.gate_activation(h, beta, eps), ref, rtol=1e-13, atol=1e-15)


def test_extremes_do_not_overflow(oracle):
    beta = np.array([2.0, 2.0, 0.5])
    h = np.array([600.0, -600.0, 4000.0])           # z = 1200, -1200, 2000: exp(z) overflows
    a = oracle.gate_activation(h, beta, 0.0)
    assert np.isfinite(a).all()
    assert a[0] == pytest.approx(600.0, rel=1e-15)  # softplus(z) -> z, alpha -> h
    assert a[1] >= 0.0 and a[1] < 1e-300
    assert a[2] == pytest.approx(4000.0, rel=1e-15)


def test_positive_and_monotone_in_h(oracle):
    h = np.linspace(-20, 20, 401)
    for b in (0.1, 1.0, 7.0):
        a = oracle.gate_activation(h, np.full_like(h, b), 1e-6)
        # 1 + exp(z) rounds to 1 below z ~ -36.7, where the form of Alg. 1 returns exactly 0
        assert (a >= 0).all() and (np.diff(a) >= 0).all()
        live = b * h > -30
        assert (a[live] > 0).all()
        assert (np.diff(a[live]) > 0).all()


def test_amplitude_limits(oracle):
    # beta -> infinity sharpens softplus(beta h)/beta into relu(h); beta -> 0+ gives ln2/beta growth
    h = np.array([-2.0, -0.5, 0.5, 2.0])
    a = oracle.gate_activation(h, np.full_like(h, 1e4), 0.0)
    np.testing.assert_allclose(a, np.maximum(h, 0.0), atol=1e-4)
    a = oracle.gate_activation(h, np.full_like(h, 1e-8), 0.0)
    np.testing.assert_allclose(a * 1e-8, np.log(2.0), rtol=1e-6)


def test_epsilon_only_scales(oracle):
    rng = np.random.default_rng(2)
    h, beta = rng.normal(size=50), rng.uniform(0.2, 3.0, size=50)
    a0 = oracle.gate_activation(h, beta, 0.0)
    a1 = oracle.gate_activation(h, beta, 0.25)
    np.testing.assert_allclose(a1 * (beta + 0.25), a0 * beta, rtol=1e-14)


def test_backward_matches_finite_differences(oracle):
    rng = np.random.default_rng(3)
    n = 200
    h = rng.normal(size=n) * 2
    beta = rng.uniform(0.2, 3.0, size=n)
    eps = 1e-3
    g = rng.normal(size=n)
    dh, dbeta = oracle.gate_activation_backward(h, beta, eps, g)
    d = 1e-6
    fh = (oracle.gate_activation(h + d, beta, eps) - oracle.gate_activation(h - d, beta, eps)) / (2 * d)
    fb = (oracle.gate_activation(h, beta + d, eps) - oracle.gate_activation(h, beta - d, eps)) / (2 * d)
    np.testing.assert_allclose(dh, g * fh, rtol=1e-7, atol=1e-9)
    np.testing.assert_allclose(dbeta, g * fb, rtol=1e-7, atol=1e-9)


def test_backward_closed_form_at_zero(oracle):
    # h = 0: sigma = 1/2, softplus = ln 2
    beta, eps = np.array([2.0]), 0.5
    dh, dbeta = oracle.gate_activation_backward(np.array([0.0]), beta, eps, np.array([1.0]))
    assert dh[0] == pytest.approx(0.5 * 2.0 / 2.5, rel=1e-15)
    assert dbeta[0] == pytest.approx(-np.log(2.0) / 2.5 ** 2, rel=1e-15)


def test_backward_extremes_are_finite(oracle):
    h = np.array([900.0, -900.0])
    beta = np.array([1.5, 1.5])
    dh, dbeta = oracle.gate_activation_backward(h, beta, 0.0, np.ones(2))
    assert np.isfinite(dh).all() and np.isfinite(dbeta).all()
    assert dh[0] == pytest.approx(1.0) and abs(dh[1]) < 1e-300
    # alpha ~ h for huge z: d alpha / d beta = h/beta - (beta h)/beta^2 = 0
    assert abs(dbeta[0]) < 1e-9


def test_chain_with_the_prefix(oracle):
    rng = np.random.default_rng(4)
    h = rng.normal(size=(1, 2, 300))
    beta = rng.uniform(0.5, 2.0, size=(1, 2, 300))
    alpha = oracle.gate_activation(h, beta, 1e-6)
    c = oracle.gate_prefix(alpha)
    np.testing.assert_allclose(c[..., -1], alpha.sum(-1), rtol=1e-13)
    assert (np.diff(c, axis=-1) > 0).all()
