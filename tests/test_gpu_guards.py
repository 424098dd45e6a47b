"""Memory safety and determinism of every entry point on the GPU, at ragged sizes.

Each output and each workspace is carved out of a larger poisoned allocation; after the call the bytes in
front of and behind it must still hold the poison (no kernel writes outside what the header says it owns).
Each call is also run twice on the same inputs and must return the same bits (no atomics, no
order-dependent reductions anywhere in the library).
"""
import numpy as np
import pytest
import torch

import gfwa_inputs as gi

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
PAD = 8192          # bytes of poison on either side
POISON = 0xA5


@pytest.fixture(scope="module")
def g():
    import paper_2512_07782_amd as mod
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    mod.load_library()
    return mod


class Guarded:
    """A tensor of `shape`/`dtype` in the middle of a poisoned byte buffer (256-byte aligned start)."""

    def __init__(self, shape, dtype):
        n = int(np.prod(shape)) * torch.empty((), dtype=dtype).element_size()
        self.n = n
        self.buf = torch.full((PAD + n + PAD,), POISON, dtype=torch.uint8, device=DEV)
        assert (self.buf.data_ptr() + PAD) % 256 == 0
        self.t = self.buf[PAD:PAD + n].view(dtype).view(shape)

    def intact(self):
        return bool((self.buf[:PAD] == POISON).all()) and bool((self.buf[PAD + self.n:] == POISON).all())

    def written(self):
        return not bool((self.buf[PAD:PAD + self.n] == POISON).all())


def dev(x, dtype):
    t = torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


SHAPES = [  # B, H, Hkv, N, d, w: ragged in every tile size the kernels use
    (1, 2, 2, 333, 128, 50), (2, 4, 2, 77, 64, 200), (1, 1, 1, 1, 128, 1), (1, 3, 1, 1027, 128, 1024),
    (1, 2, 1, 259, 64, 64), (2, 4, 2, 1301, 64, 300),   # (the last and the fourth: large enough for the fp32 matrix-core kernels)
]


@pytest.mark.parametrize("fast", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,H,Hkv,N,d,w", SHAPES)
def test_forward_backward_stay_inside_their_buffers(g, B, H, Hkv, N, d, w, dtype, fast):
    if fast and (dtype != "bf16" or d != 128):
        pytest.skip("one workspace size for this shape")
    print("guards fwd/bwd", B, H, Hkv, N, d, w, dtype, "fast" if fast else "min", flush=True)
    wl = gi.custom("guard", B, H, N, d, w, dtype, alpha_mu=-1.0, index=17, backward=True, kv_heads=Hkv)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    Q, K, V, dO = (dev(gi.make_tensor(wl, t), dtype) for t in ("Q", "K", "V", "dO"))
    alpha = dev(gi.make_tensor(wl, "alpha"), "f32")
    size = g.gfwa_backward_fast_workspace_bytes if fast else g.gfwa_backward_workspace_bytes
    results = []
    for rep in range(2):
        c = Guarded((B, H, N), torch.float32)
        O, L = Guarded((B, H, N, d), tdt), Guarded((B, H, N), torch.float32)
        dQ, dK, dV = Guarded((B, H, N, d), tdt), Guarded((B, Hkv, N, d), tdt), Guarded((B, Hkv, N, d), tdt)
        dal = Guarded((B, H, N), torch.float32)
        ws = Guarded((size(tdt, B, H, N, d, w),), torch.uint8)
        g.gfwa_gate_prefix(alpha, c.t)
        g.gfwa_forward_gqa(Q, K, V, c.t, w, wl.scale, O=O.t, L=L.t)
        g.gfwa_backward_gqa(Q, K, V, O.t, dO, c.t, L.t, w, wl.scale, workspace=ws.t, dQ=dQ.t, dK=dK.t, dV=dV.t,
                            dalpha=dal.t)
        torch.cuda.synchronize()
        for name, gd in (("c", c), ("O", O), ("L", L), ("dQ", dQ), ("dK", dK), ("dV", dV), ("dalpha", dal),
                         ("workspace", ws)):
            assert gd.intact(), f"{name}: bytes outside the buffer were written"
            assert gd.written(), f"{name}: nothing was written"
        for gd in (c, O, L, dQ, dK, dV, dal):
            assert torch.isfinite(gd.t.float()).all()
        results.append([x.t.clone() for x in (c, O, L, dQ, dK, dV, dal)])
    for a, b in zip(*results):
        assert torch.equal(a, b), "two runs on the same inputs differ"


@pytest.mark.parametrize("B,H,N", [(2, 3, 37), (1, 2, 4099), (3, 1, 20487), (1, 8, 70001)])
def test_gate_kernels_stay_inside_their_buffers(g, B, H, N):
    print("guards gate", B, H, N, flush=True)
    wl = gi.custom("guardg", B, H, N, 64, 8, alpha_mu=-1.0, index=18)
    h, beta = (dev(x, "f32") for x in gi.make_gate_inputs(wl))
    dal = dev(gi.normal(wl.seed("dO"), (B, H, N)).astype(np.float32), "f32")
    results = []
    for rep in range(2):
        outs = {k: Guarded((B, H, N), torch.float32) for k in ("c_plain", "c_act", "c_stp", "c_stp_act", "dh", "dbeta")}
        ws = Guarded((g.gfwa_gate_scan_workspace_bytes(B, H, N),), torch.uint8)
        g.gfwa_gate_prefix(h, outs["c_plain"].t)
        g.gfwa_gate_activation_prefix(h, beta, 1e-6, outs["c_act"].t)
        g.gfwa_gate_prefix_stp(h, c=outs["c_stp"].t, workspace=ws.t)
        g.gfwa_gate_prefix_stp(h, beta, 1e-6, c=outs["c_stp_act"].t, workspace=ws.t)
        g.gfwa_gate_activation_backward(h, beta, 1e-6, dal, dh=outs["dh"].t, dbeta=outs["dbeta"].t)
        torch.cuda.synchronize()
        for name, gd in list(outs.items()) + [("workspace", ws)]:
            assert gd.intact(), f"{name}: bytes outside the buffer were written"
        for name, gd in outs.items():
            assert gd.written(), name
        results.append([outs[k].t.clone() for k in sorted(outs)])
    for a, b in zip(*results):
        assert torch.equal(a, b), "two runs on the same inputs differ"


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("B,H,Hkv,T,d,w", [(3, 8, 2, 301, 128, 64), (2, 4, 1, 1003, 64, 333), (5, 6, 6, 777, 128, 2000),
                                           (1, 1, 1, 1, 64, 1)])
def test_decode_stays_inside_its_buffers(g, B, H, Hkv, T, d, w, dtype):
    print("guards decode", B, H, Hkv, T, d, w, dtype, flush=True)
    wl = gi.custom("guardd", B, H, T, d, w, dtype, alpha_mu=-1.0, index=19, kv_heads=Hkv)
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    Kc, Vc = (dev(gi.make_tensor(wl, t), dtype) for t in ("K", "V"))
    q = dev(np.ascontiguousarray(gi.make_tensor(wl, "Q")[:, :, 0, :]), dtype)
    alpha = gi.make_tensor(wl, "alpha")
    c_host = np.cumsum(alpha.astype(np.float64), axis=-1).astype(np.float32)
    pos_host = np.random.default_rng(19).integers(0, T, size=B).astype(np.int32)
    pos_host[0] = T - 1
    pos = dev(pos_host, "i32")
    a_t = dev(np.ascontiguousarray(alpha[np.arange(B), :, pos_host]), "f32")
    results = []
    for rep in range(2):
        for static in (False, True):
            c = Guarded((B, H, T), torch.float32)
            c.t.copy_(torch.from_numpy(c_host).to(DEV))
            o, L = Guarded((B, H, d), tdt), Guarded((B, H), torch.float32)
            ws = Guarded((g.gfwa_decode_workspace_bytes(B, H, T, d, w),), torch.uint8)
            if static:
                g.gfwa_decode_static(q, Kc, Vc, c.t, pos, w, wl.scale, o.t, L.t, alpha_t=a_t)
            else:
                g.gfwa_decode(q, Kc, Vc, c.t, pos, w, wl.scale, alpha_t=a_t, o=o.t, L=L.t, workspace=ws.t)
            torch.cuda.synchronize()
            for name, gd in (("c", c), ("o", o), ("L", L), ("workspace", ws)):
                assert gd.intact(), f"{name}: bytes outside the buffer were written"
            assert o.written() and L.written()
            # the cached prefix: only entry pos[b] of every (b, h) row may have changed
            changed = (c.t != torch.from_numpy(c_host).to(DEV))
            allowed = torch.zeros_like(changed)
            allowed[torch.arange(B, device=DEV), :, pos.long()] = True
            assert not bool((changed & ~allowed).any())
            results.append((o.t.clone(), L.t.clone(), c.t.clone()))
    first = results[0]
    for other in results[1:]:
        for a, b in zip(first, other):
            assert torch.equal(a, b), "runs on the same inputs differ"
