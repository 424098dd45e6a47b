"""Pins for the CPU oracle's backward pass (no GPU).

The gradients are checked against central finite differences of the oracle's own forward
(which test_oracle_forward.py pins independently), against the textbook softmax-attention
backward for a zero gate, and against identities that hold for any input.
"""
import numpy as np
import pytest
from scipy.special import softmax

RNG = np.random.default_rng(7782)


def rand_case(N, d, rng=RNG):
    Q = rng.standard_normal((N, d))
    K = rng.standard_normal((N, d))
    V = rng.standard_normal((N, d))
    alpha = np.log1p(np.exp(rng.standard_normal(N)))
    dO = rng.standard_normal((N, d))
    return Q, K, V, alpha, dO


def loss(oracle, Q, K, V, alpha, dO, w, scale):
    O, _, _ = oracle.forward(Q, K, V, alpha, w, scale)
    return float((O * dO).sum())


@pytest.mark.parametrize("N,d,w", [(24, 5, 7), (17, 3, 1), (20, 4, 20), (19, 4, 50), (33, 2, 16)])
def test_P13_finite_differences(oracle, N, d, w):
    """d/dx of sum(O * dO) for every input, including alpha (which shifts all later c)."""
    Q, K, V, alpha, dO = rand_case(N, d)
    scale = 0.41
    g = oracle.backward(Q, K, V, alpha, dO, w, scale)
    h = 1e-6
    rng = np.random.default_rng(N * 1000 + w)
    for name, X, G in (("Q", Q, g["dQ"]), ("K", K, g["dK"]), ("V", V, g["dV"])):
        for _ in range(12):
            t, x = rng.integers(N), rng.integers(d)
            Xp, Xm = X.copy(), X.copy()
            Xp[t, x] += h
            Xm[t, x] -= h
            args_p = {"Q": Q, "K": K, "V": V}
            args_m = dict(args_p)
            args_p[name], args_m[name] = Xp, Xm
            fd = (loss(oracle, args_p["Q"], args_p["K"], args_p["V"], alpha, dO, w, scale)
                  - loss(oracle, args_m["Q"], args_m["K"], args_m["V"], alpha, dO, w, scale)) / (2 * h)
            assert abs(fd - G[t, x]) <= 1e-6 * max(1.0, abs(G[t, x])), (name, t, x, fd, G[t, x])
    for q in range(N):
        ap, am = alpha.copy(), alpha.copy()
        ap[q] += h
        am[q] -= h
        fd = (loss(oracle, Q, K, V, ap, dO, w, scale) - loss(oracle, Q, K, V, am, dO, w, scale)) / (2 * h)
        assert abs(fd - g["dalpha"][q]) <= 1e-6 * max(1.0, abs(g["dalpha"][q])), (q, fd, g["dalpha"][q])


def test_P13_dc_by_finite_differences(oracle):
    """Gradient w.r.t. the prefix c itself (the quantity the two backward kernels produce)."""
    N, d, w, scale = 21, 4, 6, 0.5
    Q, K, V, alpha, dO = rand_case(N, d)
    c = oracle.gate_prefix(alpha)
    g = oracle.backward_from_c(Q, K, V, c, dO, w, scale)
    h = 1e-6
    for p in range(N):
        cp, cm = c.copy(), c.copy()
        cp[p] += h
        cm[p] -= h
        Op, _ = oracle.forward_from_c(Q, K, V, cp, w, scale)
        Om, _ = oracle.forward_from_c(Q, K, V, cm, w, scale)
        fd = ((Op - Om) * dO).sum() / (2 * h)
        assert abs(fd - g["dc"][p]) <= 1e-6 * max(1.0, abs(g["dc"][p]))


def test_P14_identities(oracle):
    N, d, w = 64, 6, 11
    Q, K, V, alpha, dO = rand_case(N, d)
    g = oracle.backward(Q, K, V, alpha, dO, w, 0.4, return_dS=True)
    dS = g["dS"]
    scale_mag = np.abs(dS).sum(axis=1).max()
    # a row-constant shift of the logits cancels in softmax: every row of dS sums to zero
    assert np.abs(dS.sum(axis=1)).max() <= 1e-12 * max(1.0, scale_mag)
    assert abs(g["dc"].sum()) <= 1e-12 * max(1.0, np.abs(g["dc"]).sum())
    # alpha_0 is part of every c_t and therefore cancels in every difference
    assert abs(g["dalpha"][0]) <= 1e-12 * max(1.0, np.abs(g["dalpha"]).max())


@pytest.mark.parametrize("N,w", [(30, 7), (25, 1), (16, 16), (12, 40)])
def test_P15_two_formulas_for_dalpha(oracle, N, w):
    Q, K, V, alpha, dO = rand_case(N, 4)
    g = oracle.backward(Q, K, V, alpha, dO, w, 0.5, return_dS=True)
    direct = oracle.dalpha_direct(g["dS"], w)
    np.testing.assert_allclose(g["dalpha"], direct, rtol=1e-11, atol=1e-13)


@pytest.mark.parametrize("w", [28, 5])
def test_P16_zero_gate_is_textbook_attention_backward(oracle, w):
    N, d, scale = 28, 6, 1 / np.sqrt(6)
    Q, K, V, _, dO = rand_case(N, d)
    g = oracle.backward(Q, K, V, np.zeros(N), dO, w, scale)
    t = np.arange(N)[:, None]
    j = np.arange(N)[None, :]
    S = np.where((j <= t) & (j > t - w), scale * Q @ K.T, -np.inf)
    P = softmax(S, axis=1)
    dP = dO @ V.T
    dS = P * (dP - (dP * P).sum(axis=1, keepdims=True))
    np.testing.assert_allclose(g["dV"], P.T @ dO, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(g["dQ"], scale * dS @ K, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(g["dK"], scale * dS.T @ Q, rtol=1e-11, atol=1e-13)
    np.testing.assert_allclose(g["dc"], dS.sum(axis=0) - dS.sum(axis=1), rtol=1e-11, atol=1e-13)


def test_P17_value_gradient_conserves_upstream_mass(oracle):
    """Rows of P sum to one, so summing dV over keys gives the sum of dO over queries."""
    N, d = 50, 5
    Q, K, V, alpha, dO = rand_case(N, d)
    g = oracle.backward(Q, K, V, alpha, dO, 9, 0.3)
    np.testing.assert_allclose(g["dV"].sum(axis=0), dO.sum(axis=0), rtol=1e-12, atol=1e-13)


def test_w1_gradients(oracle):
    """w = 1: O = V, so dV = dO and nothing else receives gradient."""
    N, d = 15, 4
    Q, K, V, alpha, dO = rand_case(N, d)
    g = oracle.backward(Q, K, V, alpha, dO, 1, 0.5)
    np.testing.assert_allclose(g["dV"], dO, rtol=1e-14)
    for k in ("dQ", "dK", "dalpha"):
        assert np.abs(g[k]).max() <= 1e-13


def test_batched_backward_shapes(oracle):
    B, H, N, d, w = 2, 2, 18, 3, 5
    rng = np.random.default_rng(5)
    Q, K, V, dO = (rng.standard_normal((B, H, N, d)) for _ in range(4))
    alpha = np.abs(rng.standard_normal((B, H, N)))
    g = oracle.backward(Q, K, V, alpha, dO, w, 0.5)
    assert g["dQ"].shape == (B, H, N, d) and g["dalpha"].shape == (B, H, N)
    g01 = oracle.backward(Q[0, 1], K[0, 1], V[0, 1], alpha[0, 1], dO[0, 1], w, 0.5)
    np.testing.assert_allclose(g["dK"][0, 1], g01["dK"], rtol=1e-13, atol=1e-15)
    np.testing.assert_allclose(g["dalpha"][0, 1], g01["dalpha"], rtol=1e-13, atol=1e-15)


# ---- Alg. 3 evaluated on a given (e.g. storage-rounded) forward output -----------------------------
def band_to_dense(Pb, N, w):
    P = np.zeros((N, N))
    for t in range(N):
        lo = max(0, t - w + 1)
        P[t, lo:t + 1] = Pb[t, :t - lo + 1]
    return P


@pytest.mark.parametrize("N,d,w", [(2, 8, 2), (2, 4, 9), (23, 6, 5), (30, 3, 64)])
def test_P19_saved_output_variant(oracle, N, d, w):
    """backward_from_c(O_saved=...) (App. E.2, Alg. 3: D = rowsum(dO * O) on the saved O).
    (a) on the exact output it is the gradient, bit for bit;
    (b) on a perturbed output the difference to the gradient is the closed form that follows from
        dS_ti = P_ti (dP_ti - D_t):  with e_t = <dO_t, O_saved_t - O_t>,
        dQ -= scale * diag(e) P K,  dK -= scale * (diag(e) P)^T Q,  dV unchanged,
        dc_p -= sum_t e_t P_tp - e_p   (written here with dense numpy matrices);
    (c) the row sums of dS then equal -e_t instead of 0, and sum_p dc_p stays 0."""
    Q, K, V, alpha, dO = rand_case(N, d, np.random.default_rng(100 * N + w))
    scale = 0.37
    c = oracle.gate_prefix(alpha)
    O, _, Pb = oracle.forward_from_c(Q, K, V, c, w, scale, return_P=True)
    g = oracle.backward_from_c(Q, K, V, c, dO, w, scale, return_dS=True)
    g0 = oracle.backward_from_c(Q, K, V, c, dO, w, scale, return_dS=True, O_saved=O)
    for k in g:
        np.testing.assert_array_equal(g[k], g0[k])
    Os = O + 0.01 * np.random.default_rng(5).standard_normal(O.shape)
    gs = oracle.backward_from_c(Q, K, V, c, dO, w, scale, return_dS=True, O_saved=Os)
    P = band_to_dense(Pb, N, w)
    e = ((Os - O) * dO).sum(axis=1)
    eP = e[:, None] * P
    np.testing.assert_allclose(gs["dQ"], g["dQ"] - scale * eP @ K, rtol=0, atol=1e-12)
    np.testing.assert_allclose(gs["dK"], g["dK"] - scale * eP.T @ Q, rtol=0, atol=1e-12)
    np.testing.assert_array_equal(gs["dV"], g["dV"])
    np.testing.assert_allclose(gs["dc"], g["dc"] - (eP.sum(axis=0) - e), rtol=0, atol=1e-12)
    np.testing.assert_allclose(gs["dS"].sum(axis=-1), -e, rtol=0, atol=1e-12)
    assert abs(gs["dc"].sum()) <= 1e-12
    assert abs(gs["dalpha"][0]) <= 1e-12
    # and the telescoped form of d(alpha) holds for this dS as for any other
    np.testing.assert_allclose(oracle.dalpha_direct(gs["dS"], w), gs["dalpha"], rtol=0, atol=1e-12)


def test_P19_rounded_output_explains_tiny_sequence_errors(oracle):
    """Storing O in bf16 perturbs D_t by up to 2^-9 sum_x |dO_tx O_tx|; when a whole gradient tensor
    rests on one or two dS entries (N = 2: dS_10 = -dS_11 is the only non-zero pair) nothing averages
    that out, and Alg. 3 on the stored output is about one per cent away from the gradient."""
    import gfwa_inputs as gi
    wl = gi.custom("fz", 1, 1, 2, 64, 2, "bf16", alpha_mu=0.5, index=31, backward=True)
    ins = {t: gi.make_tensor(wl, t)[0, 0] for t in ("Q", "K", "V", "alpha", "dO")}
    c = oracle.gate_prefix(ins["alpha"])
    O, _ = oracle.forward_from_c(ins["Q"], ins["K"], ins["V"], c, wl.w, wl.scale)
    g = oracle.backward_from_c(ins["Q"], ins["K"], ins["V"], c, ins["dO"], wl.w, wl.scale)
    gs = oracle.backward_from_c(ins["Q"], ins["K"], ins["V"], c, ins["dO"], wl.w, wl.scale,
                                O_saved=gi.round_to_bf16(O))
    r = np.linalg.norm(gs["dQ"] - g["dQ"]) / np.linalg.norm(g["dQ"])
    assert 5e-3 <= r <= 2e-2, r
    bound = 2.0 ** -9 * np.abs(ins["dO"] * O).sum(axis=1)          # |D_saved - D| per row, worst case
    assert (np.abs(((gi.round_to_bf16(O) - O) * ins["dO"]).sum(axis=1)) <= bound).all()
