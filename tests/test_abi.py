"""The C-ABI library: it loads without a GPU, exports every symbol the header declares, and
rejects bad arguments on the host before anything is launched (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2512_07782_amd as g
    return g.load_library()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gfwa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gfwa_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(lib):
    names = declared_functions()
    assert names == sorted(["gfwa_gate_prefix", "gfwa_gate_activation_prefix", "gfwa_gate_activation_backward",
                            "gfwa_forward", "gfwa_backward_workspace_bytes", "gfwa_backward_fast_workspace_bytes", "gfwa_forward_gqa", "gfwa_backward_gqa", "gfwa_decode_workspace_bytes", "gfwa_decode", "gfwa_decode_static", "gfwa_gate_scan_workspace_bytes",
                            "gfwa_gate_prefix_stp",
                            "gfwa_backward", "gfwa_strerror", "gfwa_version", "gfwa_probe_mfma", "gfwa_probe_copy", "gfwa_profile_enable",
                            "gfwa_profile_read", "gfwa_profile_kernel_name"])
    for n in names:
        assert hasattr(lib, n), n


def test_binding_exposes_the_same_names():
    import paper_2512_07782_amd as g
    for n in declared_functions():
        assert callable(getattr(g, n)), n


def test_version_and_strerror(lib):
    import paper_2512_07782_amd as g
    assert g.gfwa_version() >= 100
    assert g.gfwa_strerror(0) == "ok"
    for code in range(-6, 0):
        assert len(g.gfwa_strerror(code)) > 3
    assert "unknown" in g.gfwa_strerror(-99)


def test_argument_validation_on_host(lib):
    P = ctypes.c_void_p
    good = P(0x1000)
    odd = P(0x1004)
    f = ctypes.c_float(0.125)
    # gate prefix
    assert lib.gfwa_gate_prefix(None, good, 1, 1, 8, None) == -1
    assert lib.gfwa_gate_prefix(good, good, 0, 1, 8, None) == -2
    assert lib.gfwa_gate_prefix(good, good, 1, 1, -3, None) == -2
    assert lib.gfwa_gate_prefix(P(0x1002), good, 1, 1, 8, None) == -4
    # gate activation
    assert lib.gfwa_gate_activation_prefix(good, None, f, good, 1, 1, 8, None) == -1
    assert lib.gfwa_gate_activation_prefix(good, good, ctypes.c_float(-1.0), good, 1, 1, 8, None) == -2
    assert lib.gfwa_gate_activation_prefix(good, good, f, P(0x1002), 1, 1, 8, None) == -4
    assert lib.gfwa_gate_activation_backward(good, good, f, good, good, None, 1, 1, 8, None) == -1
    assert lib.gfwa_gate_activation_backward(good, good, f, good, good, good, 1, 0, 8, None) == -2
    # grouped-query calls: the number of key/value heads must divide the number of query heads
    assert lib.gfwa_forward_gqa(0, good, good, good, good, good, good, 1, 6, 4, 64, 128, 16, f, None) == -2
    assert lib.gfwa_forward_gqa(0, good, good, good, good, good, good, 1, 6, 0, 64, 128, 16, f, None) == -2
    assert lib.gfwa_backward_gqa(0, good, good, good, good, good, good, good, good, good, good, good, good,
                                 1 << 20, 1, 6, 5, 64, 128, 16, f, None) == -2
    # scan-then-propagate
    assert lib.gfwa_gate_prefix_stp(None, None, f, good, good, 1 << 20, 1, 1, 8, None) == -1
    assert lib.gfwa_gate_prefix_stp(good, None, f, good, None, 1 << 20, 1, 1, 8, None) == -5
    assert lib.gfwa_gate_prefix_stp(good, None, f, good, good, 0, 1, 1, 8, None) == -5
    assert lib.gfwa_gate_prefix_stp(good, good, ctypes.c_float(-1.0), good, good, 1 << 20, 1, 1, 8, None) == -2
    assert lib.gfwa_gate_scan_workspace_bytes(2, 3, 10000) == 256   # 6 rows x 3 chunks x 8 bytes, padded
    # decoding step
    dec = lambda **kw: [0, kw.get("q", good), good, good, good, None, kw.get("pos", good), good, None,
                        kw.get("ws", good), kw.get("wsb", 1 << 20), 1, kw.get("H", 4), kw.get("Hkv", 2), 64,
                        kw.get("d", 128), 16, f, None]
    assert lib.gfwa_decode(*dec(q=None)) == -1
    assert lib.gfwa_decode(*dec(pos=None)) == -1
    assert lib.gfwa_decode(*dec(Hkv=3)) == -2
    assert lib.gfwa_decode(*dec(d=96)) == -3
    assert lib.gfwa_decode(*dec(ws=None)) == -5
    assert lib.gfwa_decode(*dec(wsb=16)) == -5
    assert lib.gfwa_decode_workspace_bytes(2, 4, 1000, 128, 300) == (2 * 4 * 2 * 130 * 4 + 255) // 256 * 256   # two chunks of 256 keys
    assert lib.gfwa_decode_workspace_bytes(2, 4, 1000, 96, 300) == 0
    # the same step on the library's own scratch: argument checks, and sizes beyond its 32 MiB are refused
    decs = lambda **kw: [0, kw.get("q", good), good, good, good, None, good, good, None, kw.get("B", 1), 4,
                         kw.get("Hkv", 2), kw.get("T", 64), kw.get("d", 128), kw.get("w", 16), f, None]
    assert lib.gfwa_decode_static(*decs(q=None)) == -1
    assert lib.gfwa_decode_static(*decs(Hkv=3)) == -2
    assert lib.gfwa_decode_static(*decs(d=96)) == -3
    assert lib.gfwa_decode_static(*decs(q=odd)) == -4
    assert lib.gfwa_decode_workspace_bytes(4096, 4, 8192, 128, 8192) > 32 << 20
    assert lib.gfwa_decode_static(*decs(B=4096, T=8192, w=8192)) == -5
    # calibration kernels
    assert lib.gfwa_probe_mfma(None, 10, 256, 0, None, None) == -1
    assert lib.gfwa_probe_mfma(good, 0, 256, 1, None, None) == -2
    assert lib.gfwa_probe_copy(good, None, 1024, None) == -1
    assert lib.gfwa_probe_copy(good, good, 1000, None) == -2
    assert lib.gfwa_probe_copy(odd, good, 1024, None) == -4
    # forward
    args = lambda **kw: [kw.get("dt", 0), kw.get("Q", good), good, good, kw.get("c", good), good, good,
                         kw.get("B", 1), 2, kw.get("N", 64), kw.get("d", 128), kw.get("w", 16), f, None]
    assert lib.gfwa_forward(*args(Q=None)) == -1
    assert lib.gfwa_forward(*args(B=0)) == -2
    assert lib.gfwa_forward(*args(w=0)) == -2
    assert lib.gfwa_forward(*args(d=96)) == -3
    assert lib.gfwa_forward(*args(dt=7)) == -3
    assert lib.gfwa_forward(*args(Q=odd)) == -4
    # backward
    need = lib.gfwa_backward_workspace_bytes(0, 2, 3, 100, 64, 16)
    assert need >= 3 * 2 * 3 * 100 * 4
    assert lib.gfwa_backward_workspace_bytes(0, 2, 3, 100, 80, 16) == 0
    assert lib.gfwa_backward_workspace_bytes(0, 0, 3, 100, 64, 16) == 0
    # the faster variant's workspace: the minimum plus, for bf16 at d = 128, 2 KB per 32x32 block of the band
    # (per head: 4 query blocks of 32, each with min((16 + 30) // 32 + 1, 4) = 2 key-block slots)
    lib.gfwa_backward_fast_workspace_bytes.argtypes = lib.gfwa_backward_workspace_bytes.argtypes
    lib.gfwa_backward_fast_workspace_bytes.restype = ctypes.c_size_t
    base128 = lib.gfwa_backward_workspace_bytes(0, 2, 3, 100, 128, 16)
    assert lib.gfwa_backward_fast_workspace_bytes(0, 2, 3, 100, 128, 16) == base128 + 6 * 4 * 2 * 2048
    assert lib.gfwa_backward_fast_workspace_bytes(0, 2, 3, 100, 64, 16) == need
    assert lib.gfwa_backward_fast_workspace_bytes(1, 2, 3, 100, 128, 16) == lib.gfwa_backward_workspace_bytes(1, 2, 3, 100, 128, 16)
    assert lib.gfwa_backward_fast_workspace_bytes(0, 2, 3, 100, 128, 1 << 30) == base128 + 6 * 4 * 4 * 2048
    assert lib.gfwa_backward_fast_workspace_bytes(0, 0, 3, 100, 128, 16) == 0
    bargs = lambda **kw: [0] + [kw.get("Q", good)] + [good] * 10 + [kw.get("ws", good), kw.get("wsb", need),
                                                                   2, 3, 100, kw.get("d", 64), 16, f, None]
    assert lib.gfwa_backward(*bargs(Q=None)) == -1
    assert lib.gfwa_backward(*bargs(d=100)) == -3
    assert lib.gfwa_backward(*bargs(ws=None)) == -5
    assert lib.gfwa_backward(*bargs(wsb=need - 1)) == -5
    assert lib.gfwa_backward(*bargs(Q=odd)) == -4


def test_binding_refuses_cpu_tensors():
    import torch
    import paper_2512_07782_amd as g
    a = torch.zeros(1, 1, 8)
    with pytest.raises(ValueError):
        g.gfwa_gate_prefix(a)
