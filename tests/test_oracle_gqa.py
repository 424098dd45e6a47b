"""Pins of the oracle's grouped-query layout (query head h reads key/value head h // G).

The oracle builds it from the multi-head definition by repeating heads; the pins check that
against a dense computation written here from scratch, against finite differences through the
shared key/value heads, and against the cases that reduce to the multi-head result.
"""
import numpy as np
import pytest


def dense_gqa(Q, K, V, c, w, scale):
    """Brute force, one (b, h, t) at a time."""
    B, H, N, d = Q.shape
    G = H // K.shape[1]
    O = np.zeros_like(Q)
    L = np.zeros((B, H, N))
    for b in range(B):
        for h in range(H):
            kv = h // G
            for t in range(N):
                lo = max(0, t - w + 1)
                s = np.array([scale * Q[b, h, t] @ K[b, kv, i] - (c[b, h, t] - c[b, h, i]) for i in range(lo, t + 1)])
                m = s.max()
                e = np.exp(s - m)
                L[b, h, t] = m + np.log(e.sum())
                O[b, h, t] = (e / e.sum()) @ V[b, kv, lo:t + 1]
    return O, L


def make(rng, B, H, Hkv, N, d):
    Q, dO = rng.normal(size=(2, B, H, N, d))
    K, V = rng.normal(size=(2, B, Hkv, N, d))
    alpha = np.log1p(np.exp(rng.normal(size=(B, H, N))))
    return Q, K, V, alpha, dO


@pytest.mark.parametrize("B,H,Hkv,N,d,w", [(1, 4, 1, 9, 3, 4), (2, 6, 3, 7, 2, 100), (1, 4, 2, 12, 4, 1)])
def test_forward_matches_dense_brute_force(oracle, B, H, Hkv, N, d, w):
    rng = np.random.default_rng(10 + H)
    Q, K, V, alpha, _ = make(rng, B, H, Hkv, N, d)
    c = oracle.gate_prefix(alpha)
    O, L = oracle.forward_gqa_from_c(Q, K, V, c, w, 0.7)
    O_ref, L_ref = dense_gqa(Q, K, V, c, w, 0.7)
    np.testing.assert_allclose(O, O_ref, rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(L, L_ref, rtol=1e-12, atol=1e-13)


def test_group_of_one_is_the_multi_head_result(oracle):
    rng = np.random.default_rng(3)
    Q, K, V, alpha, dO = make(rng, 2, 3, 3, 11, 4)
    c = oracle.gate_prefix(alpha)
    O, L = oracle.forward_gqa_from_c(Q, K, V, c, 5, 0.5)
    O1, L1 = oracle.forward_from_c(Q, K, V, c, 5, 0.5)
    np.testing.assert_array_equal(O, O1)
    np.testing.assert_array_equal(L, L1)
    g = oracle.backward_gqa_from_c(Q, K, V, c, dO, 5, 0.5)
    g1 = oracle.backward_from_c(Q, K, V, c, dO, 5, 0.5)
    for k in ("dQ", "dK", "dV", "dalpha"):
        np.testing.assert_array_equal(g[k], g1[k])


def test_heads_of_a_group_with_equal_queries_and_gates_agree(oracle):
    # wrong head-to-group mapping (h % Hkv instead of h // G) would break this
    rng = np.random.default_rng(4)
    Q, K, V, alpha, _ = make(rng, 1, 4, 2, 10, 3)
    Q[:, 1], alpha[:, 1] = Q[:, 0], alpha[:, 0]      # heads 0, 1 share key/value head 0
    Q[:, 2], alpha[:, 2] = Q[:, 0], alpha[:, 0]      # head 2 reads key/value head 1
    O, _ = oracle.forward_gqa_from_c(Q, K, V, oracle.gate_prefix(alpha), 6, 1.0)
    np.testing.assert_array_equal(O[:, 0], O[:, 1])
    assert np.abs(O[:, 0] - O[:, 2]).max() > 1e-3


def test_backward_matches_finite_differences(oracle):
    rng = np.random.default_rng(5)
    B, H, Hkv, N, d, w, scale = 1, 4, 2, 8, 3, 5, 0.6
    Q, K, V, alpha, dO = make(rng, B, H, Hkv, N, d)

    def loss(Q_, K_, V_, a_):
        O, _ = oracle.forward_gqa_from_c(Q_, K_, V_, oracle.gate_prefix(a_), w, scale)
        return float((O * dO).sum())

    g = oracle.backward_gqa_from_c(Q, K, V, oracle.gate_prefix(alpha), dO, w, scale)
    assert g["dK"].shape == K.shape and g["dV"].shape == V.shape and g["dQ"].shape == Q.shape
    eps = 1e-6
    for name, X, idx in (("dQ", Q, 0), ("dK", K, 1), ("dV", V, 2), ("dalpha", alpha, 3)):
        flat = X.reshape(-1)
        for pos in rng.choice(flat.size, size=min(24, flat.size), replace=False):
            args = [Q.copy(), K.copy(), V.copy(), alpha.copy()]
            args[idx].reshape(-1)[pos] += eps
            up = loss(*args)
            args[idx].reshape(-1)[pos] -= 2 * eps
            dn = loss(*args)
            fd = (up - dn) / (2 * eps)
            an = g[name].reshape(-1)[pos]
            assert abs(fd - an) <= 1e-6 * max(1.0, abs(an)), (name, pos, fd, an)


def test_sum_of_dV_equals_sum_of_dO(oracle):
    # every row of P sums to one, whichever key/value head it reads
    rng = np.random.default_rng(6)
    Q, K, V, alpha, dO = make(rng, 2, 4, 1, 9, 3)
    g = oracle.backward_gqa_from_c(Q, K, V, oracle.gate_prefix(alpha), dO, 4, 0.9)
    np.testing.assert_allclose(g["dV"].sum(axis=(1, 2)), dO.sum(axis=(1, 2)), rtol=1e-12, atol=1e-12)
