"""gfwa_decode_static (the entry point for callers that cannot allocate: graph capture, serving loops)
against gfwa_decode through the C ABI: same kernels, so the outputs must agree bit for bit - tighter than
the parity bar of the decoding step.  Two calls in a row on the same GPU share the library's scratch array;
the second is smaller, so stale partial results of the first lie behind the part it uses."""
import ctypes

import numpy as np
import pytest
import torch

import gfwa_inputs as gi

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(x, dtype):
    t = torch.from_numpy(np.ascontiguousarray(x)).to(DEV)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def case(B, H, Hkv, T, d, w, dtype, index):
    wl = gi.custom("decs", B, H, T, d, w, dtype, alpha_mu=-1.0, index=index, kv_heads=Hkv)
    Kc, Vc, alpha = (gi.make_tensor(wl, t) for t in ("K", "V", "alpha"))
    q = np.ascontiguousarray(gi.make_tensor(wl, "Q")[:, :, 0, :])
    pos = np.random.default_rng(index).integers(0, T, size=B).astype(np.int32)
    pos[0] = T - 1
    c32 = np.cumsum(alpha.astype(np.float64), axis=-1).astype(np.float32)
    return wl, dev(q, dtype), dev(Kc, dtype), dev(Vc, dtype), dev(c32, "f32"), dev(pos, "i32")


def test_decode_static_matches_decode_on_two_calls_in_a_row():
    import paper_2512_07782_amd as g
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    lib = g.load_library()
    # first a window of five chunks with grouped heads, then a smaller problem (two chunks, then one)
    shapes = [(3, 8, 2, 1500, 128, 1200, "bf16"), (2, 4, 4, 700, 64, 300, "bf16"), (1, 2, 1, 90, 128, 64, "f32")]
    prepared = []
    for k, (B, H, Hkv, T, d, w, dtype) in enumerate(shapes):
        wl, q, Kc, Vc, c, pos = case(B, H, Hkv, T, d, w, dtype, 31 + k)
        o_ref, L_ref = g.gfwa_decode(q, Kc, Vc, c, pos, w, wl.scale)
        o = torch.full_like(q, float("nan"))
        L = torch.full((B, H), float("nan"), dtype=torch.float32, device=DEV)
        prepared.append((wl, q, Kc, Vc, c, pos, w, o, L, o_ref, L_ref))
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    for (wl, q, Kc, Vc, c, pos, w, o, L, o_ref, L_ref) in prepared:
        print("decode_static", tuple(q.shape), tuple(Kc.shape), w, flush=True)
        g.gfwa_decode_static(q, Kc, Vc, c, pos, w, wl.scale, o, L)
    assert torch.cuda.memory_allocated() == before
    torch.cuda.synchronize()
    for (wl, q, Kc, Vc, c, pos, w, o, L, o_ref, L_ref) in prepared:
        assert torch.isfinite(o.float()).all() and torch.isfinite(L).all()
        assert torch.equal(o, o_ref) and torch.equal(L, L_ref)
    # sizes beyond the library's scratch are refused on the host: nothing launched, outputs untouched
    P = ctypes.c_void_p
    big = (256, 64, 64, 8192, 128, 8192)   # 256*64 heads x 32 chunks x 130 floats = 273 MB of partials
    assert lib.gfwa_decode_workspace_bytes(big[0], big[1], big[3], big[4], big[5]) > (32 << 20)
    a = P(0x10000)
    assert lib.gfwa_decode_static(0, a, a, a, a, None, a, a, a, big[0], big[1], big[2], big[3], big[4], big[5],
                                  ctypes.c_float(0.1), None) == -5
