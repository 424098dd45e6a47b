"""Pins of the oracle's decoding step (one query against the cached window).

It must be row `pos` of the (separately pinned, C) forward oracle, reduce to textbook single-query
softmax attention without gate and window, and match the closed form for a constant gate.
"""
import numpy as np
import pytest
from scipy.special import softmax


def make(rng, B, H, Hkv, T, d):
    q = rng.normal(size=(B, H, d))
    Kc, Vc = rng.normal(size=(2, B, Hkv, T, d))
    alpha = np.log1p(np.exp(rng.normal(size=(B, H, T))))
    return q, Kc, Vc, alpha


@pytest.mark.parametrize("B,H,Hkv,T,d,w", [(2, 4, 2, 40, 8, 7), (1, 3, 3, 25, 4, 100), (3, 2, 1, 17, 5, 1)])
def test_is_the_row_of_the_forward(oracle, B, H, Hkv, T, d, w):
    rng = np.random.default_rng(20 + T)
    q, Kc, Vc, alpha = make(rng, B, H, Hkv, T, d)
    c = oracle.gate_prefix(alpha)
    pos = rng.integers(0, T, size=B)
    pos[0] = T - 1
    o, L = oracle.decode_from_c(q, Kc, Vc, c, pos, w, 0.4)
    for b in range(B):
        p = int(pos[b])
        # a sequence of length p+1 whose last query is q: rows before it do not matter
        Q = rng.normal(size=(1, H, p + 1, d))
        Q[0, :, p] = q[b]
        O_ref, L_ref = oracle.forward_gqa_from_c(Q, Kc[b:b + 1, :, :p + 1], Vc[b:b + 1, :, :p + 1],
                                                 c[b:b + 1, :, :p + 1], w, 0.4)
        np.testing.assert_allclose(o[b], O_ref[0, :, p], rtol=1e-12, atol=1e-13)
        np.testing.assert_allclose(L[b], L_ref[0, :, p], rtol=1e-12, atol=1e-13)


def test_without_gate_and_window_it_is_textbook_attention(oracle):
    rng = np.random.default_rng(7)
    q, Kc, Vc, _ = make(rng, 1, 2, 2, 30, 6)
    c = np.zeros((1, 2, 30))
    o, L = oracle.decode_from_c(q, Kc, Vc, c, [29], 1000, 0.3)
    for h in range(2):
        s = 0.3 * Kc[0, h] @ q[0, h]
        np.testing.assert_allclose(o[0, h], softmax(s) @ Vc[0, h], rtol=1e-12)
        np.testing.assert_allclose(L[0, h], np.log(np.exp(s).sum()), rtol=1e-12)


def test_constant_gate_closed_form(oracle):
    # q = 0, alpha = a: P_i = e^{-a (p - i)} (1 - e^{-a}) / (1 - e^{-a n}), n = min(p + 1, w) keys
    rng = np.random.default_rng(8)
    a, T, w, d = 0.3, 50, 12, 4
    _, Kc, Vc, _ = make(rng, 1, 1, 1, T, d)
    c = (a * np.arange(1, T + 1)).reshape(1, 1, T)
    for p in (3, 11, 12, 49):
        n = min(p + 1, w)
        o, L = oracle.decode_from_c(np.zeros((1, 1, d)), Kc, Vc, c, [p], w, 1.0)
        i = np.arange(p - n + 1, p + 1)
        P = np.exp(-a * (p - i)) * (1 - np.exp(-a)) / (1 - np.exp(-a * n))
        np.testing.assert_allclose(o[0, 0], P @ Vc[0, 0, i], rtol=1e-12)
        np.testing.assert_allclose(L[0, 0], np.log((1 - np.exp(-a * n)) / (1 - np.exp(-a))), rtol=1e-12, atol=1e-14)


def test_window_of_one_returns_the_newest_value(oracle):
    rng = np.random.default_rng(9)
    q, Kc, Vc, alpha = make(rng, 2, 2, 1, 9, 3)
    pos = [4, 8]
    o, L = oracle.decode_from_c(q, Kc, Vc, oracle.gate_prefix(alpha), pos, 1, 0.5)
    for b in range(2):
        np.testing.assert_array_equal(o[b], np.broadcast_to(Vc[b, 0, pos[b]], (2, 3)))
        np.testing.assert_allclose(L[b], 0.5 * q[b] @ Kc[b, 0, pos[b]], rtol=1e-13)


def test_positions_past_the_query_are_not_read(oracle):
    rng = np.random.default_rng(11)
    q, Kc, Vc, alpha = make(rng, 1, 2, 2, 20, 3)
    c = oracle.gate_prefix(alpha)
    o1, L1 = oracle.decode_from_c(q, Kc, Vc, c, [10], 6, 0.5)
    Kc[:, :, 11:], Vc[:, :, 11:], c[:, :, 11:] = np.nan, np.nan, np.nan
    Kc[:, :, :5], Vc[:, :, :5] = np.nan, np.nan      # and neither are positions before the window
    o2, L2 = oracle.decode_from_c(q, Kc, Vc, c, [10], 6, 0.5)
    np.testing.assert_array_equal(o1, o2)
    np.testing.assert_array_equal(L1, L2)
