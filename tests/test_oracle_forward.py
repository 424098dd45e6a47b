"""Pins for the CPU oracle's forward pass and gate prefix (no GPU).

Each test checks the oracle against something the paper or the mathematics fixes
independently of the oracle's own code: a dense brute force written here, textbook
special cases (Sec. 3, the causal-softmax and sliding-window scores defined after
Eq. 1), closed forms, invariants, and a hand-worked example under tests/golden/.
"""
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy.special import logsumexp, softmax

RNG = np.random.default_rng(20251207)
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand_case(N, d, w_unused=None, alpha_scale=1.0, rng=RNG):
    Q = rng.standard_normal((N, d))
    K = rng.standard_normal((N, d))
    V = rng.standard_normal((N, d))
    alpha = alpha_scale * np.log1p(np.exp(rng.standard_normal(N)))
    return Q, K, V, alpha


def dense_brute_force(Q, K, V, alpha, w, scale):
    """Explicit N x N logits with -inf outside the window, then row softmax (Sec. 3.2)."""
    N = Q.shape[0]
    u = -np.cumsum(alpha)                         # the paper's u_t
    Phi = scale * (Q @ K.T)
    Bias = u[:, None] - u[None, :]                # B_tj = u_t - u_j
    t = np.arange(N)[:, None]
    j = np.arange(N)[None, :]
    keep = (j <= t) & (j > t - w)
    S = np.where(keep, Phi + Bias, -np.inf)
    P = softmax(S, axis=1)
    return P @ V, logsumexp(S, axis=1), P


def band_to_dense(P_band, w):
    N, wb = P_band.shape
    P = np.zeros((N, N))
    for t in range(N):
        lo = max(0, t - w + 1)
        P[t, lo:t + 1] = P_band[t, :t - lo + 1]
    return P


@pytest.mark.parametrize("N,d,w", [(37, 5, 1), (37, 5, 7), (64, 8, 64), (50, 3, 200), (129, 16, 33),
                                   (1, 4, 3), (2, 1, 2)])
def test_P1_dense_brute_force(oracle, N, d, w):
    Q, K, V, alpha = rand_case(N, d)
    scale = 0.37
    O, L, c = oracle.forward(Q, K, V, alpha, w, scale)
    O_ref, L_ref, P_ref = dense_brute_force(Q, K, V, alpha, w, scale)
    np.testing.assert_allclose(O, O_ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(L, L_ref, rtol=1e-12, atol=1e-13)
    _, _, P_band = oracle.forward_from_c(Q, K, V, c, w, scale, return_P=True)
    np.testing.assert_allclose(band_to_dense(P_band, w), P_ref, rtol=1e-12, atol=1e-15)


def test_P1_transposed_operand_would_fail(oracle):
    """Guard the brute force itself: swapping Q and K changes the answer."""
    Q, K, V, alpha = rand_case(20, 4)
    O, _, _ = oracle.forward(Q, K, V, alpha, 5, 0.5)
    O_sw, _, _ = dense_brute_force(K, Q, V, alpha, 5, 0.5)
    assert np.abs(O - O_sw).max() > 1e-3


def test_P2_zero_gate_is_sliding_window_attention(oracle):
    """alpha = 0 gives the sliding-window score of Sec. 3 (row-by-row textbook softmax)."""
    N, d, w, scale = 45, 6, 9, 1 / np.sqrt(6)
    Q, K, V, _ = rand_case(N, d)
    O, L, _ = oracle.forward(Q, K, V, np.zeros(N), w, scale)
    for t in range(N):
        lo = max(0, t - w + 1)
        logits = scale * (K[lo:t + 1] @ Q[t])
        np.testing.assert_allclose(O[t], softmax(logits) @ V[lo:t + 1], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(L[t], logsumexp(logits), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("w", [40, 41, 1000])
def test_P2_zero_gate_full_window_is_causal_softmax(oracle, w):
    N, d, scale = 40, 8, 1 / np.sqrt(8)
    Q, K, V, _ = rand_case(N, d)
    O, L, _ = oracle.forward(Q, K, V, np.zeros(N), w, scale)
    S = scale * Q @ K.T
    S[np.triu_indices(N, 1)] = -np.inf
    np.testing.assert_allclose(O, softmax(S, axis=1) @ V, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(L, logsumexp(S, axis=1), rtol=1e-12, atol=1e-14)


def test_P3_rows_are_distributions_on_the_window(oracle):
    N, d, w = 70, 4, 13
    Q, K, V, alpha = rand_case(N, d)
    c = oracle.gate_prefix(alpha)
    _, _, P_band = oracle.forward_from_c(Q, K, V, c, w, 0.5, return_P=True)
    assert (P_band >= 0).all()
    np.testing.assert_allclose(P_band.sum(axis=1), 1.0, rtol=0, atol=1e-14)
    for t in range(N):
        n = min(t + 1, w)
        assert (P_band[t, n:] == 0).all()          # nothing outside the window
        assert (P_band[t, :n] > 0).all()


@pytest.mark.parametrize("a", [0.05, np.log(2.0), 3.0])
def test_P4_closed_form_constant_gate_zero_queries(oracle, a):
    """Q = 0, alpha = a: weights are a truncated geometric series in the distance t - i."""
    N, d, w = 60, 3, 11
    _, K, V, _ = rand_case(N, d)
    O, L, _ = oracle.forward(np.zeros((N, d)), K, V, np.full(N, a), w, 1.0)
    r = np.exp(-a)
    for t in range(N):
        n = min(t + 1, w)
        dist = np.arange(n - 1, -1, -1)            # key i = t-n+1 .. t  ->  distance t-i
        P = r ** dist * (1 - r) / (1 - r ** n)
        np.testing.assert_allclose(O[t], P @ V[t - n + 1:t + 1], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(L[t], np.log((1 - r ** n) / (1 - r)), rtol=1e-12, atol=1e-14)


def test_P5_constant_gate_is_a_linear_distance_bias(oracle):
    """alpha = a turns the bias into -a (t - i): windowed attention with that explicit slope."""
    N, d, w, a, scale = 48, 5, 10, 0.3, 0.44
    Q, K, V, _ = rand_case(N, d)
    O, L, _ = oracle.forward(Q, K, V, np.full(N, a), w, scale)
    for t in range(N):
        lo = max(0, t - w + 1)
        idx = np.arange(lo, t + 1)
        logits = scale * (K[idx] @ Q[t]) - a * (t - idx)
        np.testing.assert_allclose(O[t], softmax(logits) @ V[idx], rtol=1e-12, atol=1e-14)
        np.testing.assert_allclose(L[t], logsumexp(logits), rtol=1e-12, atol=1e-14)


def test_P6_window_of_one(oracle):
    N, d, scale = 33, 7, 0.61
    Q, K, V, alpha = rand_case(N, d)
    O, L, _ = oracle.forward(Q, K, V, alpha, 1, scale)
    np.testing.assert_array_equal(O, V)
    np.testing.assert_allclose(L, scale * np.einsum("td,td->t", Q, K), rtol=1e-14, atol=1e-15)


def test_P7_strong_gate_keeps_only_the_current_token(oracle):
    N, d = 30, 4
    Q, K, V, _ = rand_case(N, d)
    Q *= 0.1
    O, _, _ = oracle.forward(Q, K, V, np.full(N, 50.0), 8, 0.5)
    np.testing.assert_allclose(O, V, rtol=0, atol=1e-19)


def test_P8_constant_values(oracle):
    N, d = 40, 6
    Q, K, _, alpha = rand_case(N, d)
    v = RNG.standard_normal(d)
    O, _, _ = oracle.forward(Q, K, np.tile(v, (N, 1)), alpha, 9, 0.4)
    np.testing.assert_allclose(O, np.tile(v, (N, 1)), rtol=1e-13, atol=1e-15)


def test_P9_only_prefix_differences_matter(oracle):
    N, d, w = 52, 4, 12
    Q, K, V, alpha = rand_case(N, d)
    c = oracle.gate_prefix(alpha)
    O0, L0 = oracle.forward_from_c(Q, K, V, c, w, 0.5)
    O1, L1 = oracle.forward_from_c(Q, K, V, c + 123.0, w, 0.5)
    np.testing.assert_allclose(O1, O0, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(L1, L0, rtol=1e-11, atol=1e-12)
    alpha2 = alpha.copy()
    alpha2[0] += 5.0                                # alpha_0 is in every c_t, so it cancels
    O2, L2, _ = oracle.forward(Q, K, V, alpha2, w, 0.5)
    np.testing.assert_allclose(O2, O0, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(L2, L0, rtol=1e-11, atol=1e-12)


def test_P9b_gate_direction(oracle):
    """A larger gate at position q must move weight from keys before q to keys at or after q."""
    N, d, w, q = 24, 3, 24, 10
    Q, K, V, alpha = rand_case(N, d)
    c0 = oracle.gate_prefix(alpha)
    a2 = alpha.copy()
    a2[q] += 2.0
    c1 = oracle.gate_prefix(a2)
    _, _, P0 = oracle.forward_from_c(Q, K, V, c0, w, 0.5, return_P=True)
    _, _, P1 = oracle.forward_from_c(Q, K, V, c1, w, 0.5, return_P=True)
    D0, D1 = band_to_dense(P0, w), band_to_dense(P1, w)
    for t in range(q, N):
        assert D1[t, :q].sum() < D0[t, :q].sum()
    np.testing.assert_allclose(D1[:q], D0[:q], rtol=1e-12, atol=1e-15)   # rows before q unaffected


def test_P10_prefix_is_nondecreasing_and_bias_nonpositive(oracle):
    alpha = np.log1p(np.exp(RNG.standard_normal((3, 2, 100))))
    c = oracle.gate_prefix(alpha)
    assert c.shape == alpha.shape
    assert (np.diff(c, axis=-1) >= 0).all()
    assert (c >= 0).all()


def test_P11_L_reconstructs_P(oracle):
    """Alg. 3 rebuilds p = exp(S - L): the oracle's L must do that for the oracle's P."""
    N, d, w, scale = 41, 5, 8, 0.47
    Q, K, V, alpha = rand_case(N, d)
    c = oracle.gate_prefix(alpha)
    _, L, P_band = oracle.forward_from_c(Q, K, V, c, w, scale, return_P=True)
    for t in range(N):
        lo = max(0, t - w + 1)
        S = scale * (K[lo:t + 1] @ Q[t]) + (c[lo:t + 1] - c[t])
        np.testing.assert_allclose(np.exp(S - L[t]), P_band[t, :t - lo + 1], rtol=1e-12, atol=1e-16)


def test_P12_gate_prefix(oracle):
    alpha = np.abs(RNG.standard_normal((2, 3, 1000)))
    c = oracle.gate_prefix(alpha)
    np.testing.assert_allclose(c, np.cumsum(alpha, axis=-1), rtol=1e-13)
    np.testing.assert_allclose(c[..., -1], alpha.sum(axis=-1), rtol=1e-13)
    ones = oracle.gate_prefix(np.ones(5000))
    np.testing.assert_array_equal(ones, np.arange(1, 5001, dtype=np.float64))
    # inclusive, not exclusive
    assert oracle.gate_prefix(np.array([2.0, 3.0]))[0] == 2.0


def test_golden_half_life_example(oracle):
    rows = []
    with open(os.path.join(GOLDEN, "half_life_example.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            t, v, o, el = line.split()
            rows.append((int(t), float(v), float(Fraction(o)), float(Fraction(el))))
    N = len(rows)
    V = np.array([[r[1]] for r in rows])
    O, L, _ = oracle.forward(np.zeros((N, 1)), np.zeros((N, 1)), V, np.full(N, np.log(2.0)), 2, 1.0)
    np.testing.assert_allclose(O[:, 0], [r[2] for r in rows], rtol=1e-14)
    np.testing.assert_allclose(np.exp(L), [r[3] for r in rows], rtol=1e-14)


def test_batched_shapes(oracle):
    B, H, N, d, w = 2, 3, 20, 4, 6
    Q = RNG.standard_normal((B, H, N, d))
    K = RNG.standard_normal((B, H, N, d))
    V = RNG.standard_normal((B, H, N, d))
    alpha = np.abs(RNG.standard_normal((B, H, N)))
    O, L, c = oracle.forward(Q, K, V, alpha, w, 0.5)
    assert O.shape == (B, H, N, d) and L.shape == (B, H, N) and c.shape == (B, H, N)
    O11, L11, _ = dense_brute_force(Q[1, 1], K[1, 1], V[1, 1], alpha[1, 1], w, 0.5)
    np.testing.assert_allclose(O[1, 1], O11, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(L[1, 1], L11, rtol=1e-12, atol=1e-14)
