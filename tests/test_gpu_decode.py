"""Parity of the decoding step (gfwa_decode, through the C ABI) with the oracle's decode_from_c.

Inputs: seeded caches of the workload generators' value distributions; positions mix short
prefixes (window clipped at 0), positions inside the cache and the last slot.
Bars: bf16 |o - ref| <= 2e-2 max, 2e-3 mean (the forward's), fp32 1e-5 relative; L as the forward's
(1e-4 + 1e-5 |L| + 2^-21 times the largest gate difference over a window).
"""
import numpy as np
import pytest
import torch

import gfwa_inputs as gi

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


@pytest.fixture(scope="module")
def g():
    import paper_2512_07782_amd as mod
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    mod.load_library()
    return mod


def dev(x, dtype):
    t = torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def host(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


def window_span(c, w):
    """Largest gate difference that enters any logit: max_t c_t - c_{max(0, t-w+1)} (c non-decreasing)."""
    c = np.asarray(c, dtype=np.float64)
    N = c.shape[-1]
    r = min(N - 1, int(w) - 1)
    return float((c[..., r:] - c[..., :N - r]).max()) if r > 0 else 0.0


def make_case(B, H, Hkv, T, d, w, dtype, index):
    wl = gi.custom("dec", B, H, T, d, w, dtype, alpha_mu=-1.0, index=index, kv_heads=Hkv)
    Kc, Vc, alpha = (gi.make_tensor(wl, t) for t in ("K", "V", "alpha"))
    q = gi.make_tensor(wl, "Q")[:, :, 0, :]                       # [B,H,d], already rounded to the storage type
    rng = np.random.default_rng(index)
    pos = rng.integers(0, T, size=B).astype(np.int32)
    pos[0] = T - 1
    if B > 1:
        pos[1] = min(T - 1, 3)
    return wl, np.ascontiguousarray(q), Kc, Vc, alpha, pos


CASES = [
    # B, H, Hkv, T, d, w
    (1, 1, 1, 1, 64, 1), (2, 4, 4, 37, 64, 5), (3, 8, 2, 300, 128, 64), (2, 4, 1, 1000, 128, 333),
    (4, 6, 3, 777, 64, 2000), (2, 3, 3, 1500, 128, 1024), (5, 16, 4, 4099, 128, 1024), (2, 8, 8, 600, 64, 257),
]


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,H,Hkv,T,d,w", CASES)
def test_decode_matches_oracle(g, oracle, B, H, Hkv, T, d, w, dtype):
    print("decode", B, H, Hkv, T, d, w, dtype, flush=True)
    wl, q, Kc, Vc, alpha, pos = make_case(B, H, Hkv, T, d, w, dtype, 21)
    c32 = oracle.gate_prefix(alpha).astype(np.float32)
    o, L = g.gfwa_decode(dev(q, dtype), dev(Kc, dtype), dev(Vc, dtype), dev(c32, "f32"), dev(pos, "i32"), w, wl.scale)
    torch.cuda.synchronize()
    o_ref, L_ref = oracle.decode_from_c(q, Kc, Vc, c32, pos, w, wl.scale)
    err = np.abs(host(o) - o_ref)
    lerr = np.abs(host(L) - L_ref)
    print(f"  o max {err.max():.3e} mean {err.mean():.3e}  L max {lerr.max():.3e}", flush=True)
    if dtype == "bf16":
        assert err.max() <= 2e-2 and err.mean() <= 2e-3
    else:
        assert err.max() <= 1e-5 * np.abs(o_ref).max()
    assert (lerr <= 1e-4 + 1e-5 * np.abs(L_ref) + 2.0 ** -21 * window_span(c32, w)).all()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,H,Hkv,T,d,w", [(2, 8, 2, 700, 128, 512), (2, 4, 2, 900, 64, 300), (1, 4, 4, 640, 128, 640)])
def test_decode_with_scores_far_apart(g, oracle, B, H, Hkv, T, d, w, dtype):
    # queries and keys of large norm: scores differ by far more than 2^60 inside a wave's 64 keys, so the
    # exponentials cannot all be taken against the score of the newest key (the reference must be raised)
    wl = gi.custom("decbig", B, H, T, d, w, dtype, alpha_mu=-1.0, index=25, kv_heads=Hkv, qkv_std=4.0)
    Kc, Vc, alpha = (gi.make_tensor(wl, t) for t in ("K", "V", "alpha"))
    q = np.ascontiguousarray(gi.make_tensor(wl, "Q")[:, :, 0, :])
    # one early key of the window aligned with the query of head 0: by far the largest score
    pos = np.full(B, T - 1, dtype=np.int32)
    Kc[:, 0, T - 40, :] = q[:, 0, :]
    c32 = oracle.gate_prefix(alpha).astype(np.float32)
    o, L = g.gfwa_decode(dev(q, dtype), dev(Kc, dtype), dev(Vc, dtype), dev(c32, "f32"), dev(pos, "i32"), w, wl.scale)
    torch.cuda.synchronize()
    o_ref, L_ref = oracle.decode_from_c(q, Kc, Vc, c32, pos, w, wl.scale)
    spread = wl.scale * np.abs(np.einsum("bhd,bhd->bh", q, q)).max()
    print(f"  largest score about {spread:.0f} nats", flush=True)
    assert spread > 100
    err = np.abs(host(o) - o_ref)
    assert np.isfinite(host(o)).all() and np.isfinite(host(L)).all()
    if dtype == "bf16":
        assert err.max() <= 4 * 2e-2 and err.mean() <= 4 * 2e-3          # values are 4 times larger here
    else:
        assert err.max() <= 1e-5 * np.abs(o_ref).max()
    assert (np.abs(host(L) - L_ref) <= 1e-4 + 1e-5 * np.abs(L_ref) + 2.0 ** -21 * window_span(c32, w)).all()


@pytest.mark.parametrize("B,H,Hkv,T,d,w", [(3, 8, 2, 300, 128, 64), (2, 4, 1, 1000, 64, 333)])
def test_decode_advances_the_gate_prefix(g, oracle, B, H, Hkv, T, d, w):
    wl, q, Kc, Vc, alpha, pos = make_case(B, H, Hkv, T, d, w, "bf16", 22)
    pos[-1] = 0                                                   # a sequence at its first token
    c32 = oracle.gate_prefix(alpha).astype(np.float32)
    bi = np.arange(B)
    a_t = np.ascontiguousarray(alpha[bi, :, pos])                 # [B,H], the new token's gate
    prev = np.where(pos[:, None] > 0, c32[bi, :, np.maximum(pos - 1, 0)], np.float32(0))
    c_new = (prev.astype(np.float32) + a_t.astype(np.float32)).astype(np.float32)   # the same fp32 addition
    # cache state before the step: entry pos (and everything after it) not yet written
    c_in = c32.copy()
    for b in range(B):
        c_in[b, :, pos[b]:] = np.nan
    cd = dev(c_in, "f32")
    o, L = g.gfwa_decode(dev(q, "bf16"), dev(Kc, "bf16"), dev(Vc, "bf16"), cd, dev(pos, "i32"), w, wl.scale,
                         alpha_t=dev(a_t, "f32"))
    torch.cuda.synchronize()
    c_out = cd.cpu().numpy()
    c_exp = c32.copy()
    c_exp[bi, :, pos] = c_new
    for b in range(B):
        np.testing.assert_array_equal(c_out[b, :, pos[b]], c_new[b])             # written, bit for bit
        assert np.isnan(c_out[b, :, pos[b] + 1:]).all()                           # nothing past it touched
        np.testing.assert_array_equal(c_out[b, :, :pos[b]], c32[b, :, :pos[b]])  # nothing before it touched
    o_ref, L_ref = oracle.decode_from_c(q, Kc, Vc, np.nan_to_num(c_exp), pos, w, wl.scale)
    assert np.isfinite(host(o)).all()
    assert np.abs(host(o) - o_ref).max() <= 2e-2
    assert (np.abs(host(L) - L_ref) <= 1e-4 + 1e-5 * np.abs(L_ref) + 2.0 ** -21 * window_span(c32, w)).all()


def test_decode_agrees_with_the_forward_kernel_row(g, oracle):
    # the two GPU paths on the same data: the last row of a full forward against a decoding step
    wl = gi.custom("decfwd", 1, 8, 2048, 128, 512, "bf16", alpha_mu=-1.0, index=23, kv_heads=2)
    Q, K, V, alpha = (gi.make_tensor(wl, t) for t in ("Q", "K", "V", "alpha"))
    cd = g.gfwa_gate_prefix(dev(alpha, "f32"))
    O, L = g.gfwa_forward_gqa(dev(Q, "bf16"), dev(K, "bf16"), dev(V, "bf16"), cd, wl.w, wl.scale)
    p = wl.N - 1
    o, l = g.gfwa_decode(dev(np.ascontiguousarray(Q[:, :, p]), "bf16"), dev(K, "bf16"), dev(V, "bf16"), cd,
                         torch.full((1,), p, dtype=torch.int32, device=DEV), wl.w, wl.scale)
    torch.cuda.synchronize()
    assert np.abs(host(o) - host(O[:, :, p])).max() <= 2e-2
    assert np.abs(host(l) - host(L[:, :, p])).max() <= 1e-3


def test_decode_rows_outside_the_window_are_not_read(g, oracle):
    wl, q, Kc, Vc, alpha, pos = make_case(2, 4, 2, 500, 128, 100, "f32", 24)
    pos[:] = [250, 499]
    c32 = oracle.gate_prefix(alpha).astype(np.float32)
    o1, L1 = g.gfwa_decode(dev(q, "f32"), dev(Kc, "f32"), dev(Vc, "f32"), dev(c32, "f32"), dev(pos, "i32"), 100, wl.scale)
    Kp, Vp = Kc.copy(), Vc.copy()
    Kp[0, :, 251:], Vp[0, :, 251:] = np.nan, np.nan
    Kp[0, :, :151], Vp[0, :, :151] = np.nan, np.nan
    Kp[1, :, :400], Vp[1, :, :400] = np.nan, np.nan
    o2, L2 = g.gfwa_decode(dev(q, "f32"), dev(Kp, "f32"), dev(Vp, "f32"), dev(c32, "f32"), dev(pos, "i32"), 100, wl.scale)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(L1, L2)


def test_decode_clamps_positions_outside_the_cache(g, oracle):
    # a position below 0 or past the cache is taken as the first / last slot: nothing outside is touched
    wl, q, Kc, Vc, alpha, _ = make_case(3, 4, 2, 300, 64, 50, "f32", 27)
    c32 = oracle.gate_prefix(alpha).astype(np.float32)
    args = (dev(q, "f32"), dev(Kc, "f32"), dev(Vc, "f32"), dev(c32, "f32"))
    bad = torch.tensor([-5, 300, 1 << 30], dtype=torch.int32, device=DEV)
    good = torch.tensor([0, 299, 299], dtype=torch.int32, device=DEV)
    o1, L1 = g.gfwa_decode(*args, bad, 50, wl.scale)
    o2, L2 = g.gfwa_decode(*args, good, 50, wl.scale)
    torch.cuda.synchronize()
    assert torch.equal(o1, o2) and torch.equal(L1, L2)
