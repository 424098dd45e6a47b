"""ctypes binding with the same names as the C ABI (include/gfwa.h).

Each function takes torch tensors living on the GPU, checks shapes/dtypes/contiguity on the
host, and passes raw device pointers and the current HIP stream to the library.  There is no
fallback: if `libgfwa.so` has not been built the import of the library raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# GFWA_LIB names another build of the same library (a host-sanitizer build, for one)
_LIB_PATH = os.environ.get("GFWA_LIB") or os.path.join(_HERE, "libgfwa.so")
_lib: Optional[ctypes.CDLL] = None

GFWA_BF16, GFWA_F32 = 0, 1

EXPORTS = ("gfwa_gate_prefix", "gfwa_gate_activation_prefix", "gfwa_gate_activation_backward", "gfwa_forward", "gfwa_backward_workspace_bytes", "gfwa_backward_fast_workspace_bytes", "gfwa_backward",
           "gfwa_forward_gqa", "gfwa_backward_gqa", "gfwa_decode_workspace_bytes", "gfwa_decode", "gfwa_decode_static", "gfwa_gate_scan_workspace_bytes", "gfwa_gate_prefix_stp",
           "gfwa_strerror", "gfwa_version", "gfwa_probe_mfma", "gfwa_probe_copy", "gfwa_profile_enable", "gfwa_profile_read",
           "gfwa_profile_kernel_name")
N_KERNELS = 13


class GfwaError(RuntimeError):
    def __init__(self, code: int, text: str):
        super().__init__(f"libgfwa error {code}: {text}")
        self.code = code


def lib_path() -> str:
    return _LIB_PATH


def load_library() -> ctypes.CDLL:
    """Load libgfwa.so, building it first only if no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        from .build import build
        build()
    lib = ctypes.CDLL(_LIB_PATH)
    vp, fp, i, f = ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_float
    lib.gfwa_gate_prefix.argtypes = [fp, fp, i, i, i, vp]
    lib.gfwa_gate_prefix.restype = i
    lib.gfwa_gate_activation_prefix.argtypes = [fp, fp, ctypes.c_float, fp, i, i, i, vp]
    lib.gfwa_gate_activation_prefix.restype = i
    lib.gfwa_gate_activation_backward.argtypes = [fp, fp, ctypes.c_float, fp, fp, fp, i, i, i, vp]
    lib.gfwa_gate_activation_backward.restype = i
    lib.gfwa_forward.argtypes = [i, vp, vp, vp, fp, vp, fp, i, i, i, i, i, f, vp]
    lib.gfwa_forward.restype = i
    lib.gfwa_backward_workspace_bytes.argtypes = [i, i, i, i, i, i]
    lib.gfwa_backward_workspace_bytes.restype = ctypes.c_size_t
    lib.gfwa_backward_fast_workspace_bytes.argtypes = [i, i, i, i, i, i]
    lib.gfwa_backward_fast_workspace_bytes.restype = ctypes.c_size_t
    lib.gfwa_backward.argtypes = [i, vp, vp, vp, vp, vp, fp, fp, vp, vp, vp, fp, vp, ctypes.c_size_t,
                                  i, i, i, i, i, f, vp]
    lib.gfwa_backward.restype = i
    lib.gfwa_forward_gqa.argtypes = [i, vp, vp, vp, fp, vp, fp, i, i, i, i, i, i, f, vp]
    lib.gfwa_forward_gqa.restype = i
    lib.gfwa_backward_gqa.argtypes = [i, vp, vp, vp, vp, vp, fp, fp, vp, vp, vp, fp, vp, ctypes.c_size_t,
                                      i, i, i, i, i, i, f, vp]
    lib.gfwa_backward_gqa.restype = i
    lib.gfwa_decode_workspace_bytes.argtypes = [i, i, i, i, i]
    lib.gfwa_decode_workspace_bytes.restype = ctypes.c_size_t
    lib.gfwa_decode.argtypes = [i, vp, vp, vp, fp, fp, vp, vp, fp, vp, ctypes.c_size_t, i, i, i, i, i, i, f, vp]
    lib.gfwa_decode.restype = i
    lib.gfwa_decode_static.argtypes = [i, vp, vp, vp, fp, fp, vp, vp, fp, i, i, i, i, i, i, f, vp]
    lib.gfwa_decode_static.restype = i
    lib.gfwa_gate_scan_workspace_bytes.argtypes = [i, i, i]
    lib.gfwa_gate_scan_workspace_bytes.restype = ctypes.c_size_t
    lib.gfwa_gate_prefix_stp.argtypes = [fp, fp, f, fp, vp, ctypes.c_size_t, i, i, i, vp]
    lib.gfwa_gate_prefix_stp.restype = i
    lib.gfwa_probe_mfma.argtypes = [fp, i, i, i, ctypes.POINTER(ctypes.c_double), vp]
    lib.gfwa_probe_mfma.restype = i
    lib.gfwa_probe_copy.argtypes = [vp, vp, ctypes.c_size_t, vp]
    lib.gfwa_probe_copy.restype = i
    lib.gfwa_strerror.argtypes = [i]
    lib.gfwa_strerror.restype = ctypes.c_char_p
    lib.gfwa_version.argtypes = []
    lib.gfwa_version.restype = i
    lib.gfwa_profile_enable.argtypes = [i]
    lib.gfwa_profile_enable.restype = i
    lib.gfwa_profile_read.argtypes = [ctypes.POINTER(ctypes.c_float), ctypes.POINTER(ctypes.c_int), i]
    lib.gfwa_profile_read.restype = i
    lib.gfwa_profile_kernel_name.argtypes = [i]
    lib.gfwa_profile_kernel_name.restype = ctypes.c_char_p
    _lib = lib
    return lib


def gfwa_strerror(code: int) -> str:
    return load_library().gfwa_strerror(int(code)).decode()


def gfwa_version() -> int:
    return int(load_library().gfwa_version())


def _check(code: int) -> None:
    if code != 0:
        raise GfwaError(code, gfwa_strerror(code))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.bfloat16:
        return GFWA_BF16
    if t.dtype == torch.float32:
        return GFWA_F32
    raise TypeError(f"unsupported dtype {t.dtype}: bfloat16 or float32")


def _need(t: torch.Tensor, shape, dtype, name: str) -> None:
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU")
    if tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")
    if t.dtype != dtype:
        raise TypeError(f"{name} has dtype {t.dtype}, expected {dtype}")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")


def gfwa_gate_prefix(alpha: torch.Tensor, c: Optional[torch.Tensor] = None) -> torch.Tensor:
    """c[b,h,t] = sum_{q<=t} alpha[b,h,q];  alpha, c: [B,H,N] fp32 on the GPU."""
    if alpha.dim() != 3:
        raise ValueError("alpha must be [B,H,N]")
    B, H, N = alpha.shape
    _need(alpha, (B, H, N), torch.float32, "alpha")
    if c is None:
        c = torch.empty_like(alpha)
    _need(c, (B, H, N), torch.float32, "c")
    _check(load_library().gfwa_gate_prefix(alpha.data_ptr(), c.data_ptr(), B, H, N, _stream()))
    return c


def gfwa_gate_activation_prefix(hpre: torch.Tensor, beta: torch.Tensor, eps: float,
                                c: Optional[torch.Tensor] = None) -> torch.Tensor:
    """c = cumsum_t softplus(beta * hpre) / (beta + eps);  hpre, beta, c: [B,H,N] fp32 on the GPU."""
    if hpre.dim() != 3:
        raise ValueError("hpre must be [B,H,N]")
    B, H, N = hpre.shape
    _need(hpre, (B, H, N), torch.float32, "hpre")
    _need(beta, (B, H, N), torch.float32, "beta")
    if c is None:
        c = torch.empty_like(hpre)
    _need(c, (B, H, N), torch.float32, "c")
    _check(load_library().gfwa_gate_activation_prefix(hpre.data_ptr(), beta.data_ptr(), float(eps), c.data_ptr(),
                                                      B, H, N, _stream()))
    return c


def gfwa_gate_activation_backward(hpre: torch.Tensor, beta: torch.Tensor, eps: float, dalpha: torch.Tensor,
                                  dh: Optional[torch.Tensor] = None, dbeta: Optional[torch.Tensor] = None):
    """(dh, dbeta) from d(alpha); all [B,H,N] fp32 on the GPU."""
    if hpre.dim() != 3:
        raise ValueError("hpre must be [B,H,N]")
    B, H, N = hpre.shape
    for name, t in (("hpre", hpre), ("beta", beta), ("dalpha", dalpha)):
        _need(t, (B, H, N), torch.float32, name)
    if dh is None:
        dh = torch.empty_like(hpre)
    if dbeta is None:
        dbeta = torch.empty_like(hpre)
    _need(dh, (B, H, N), torch.float32, "dh")
    _need(dbeta, (B, H, N), torch.float32, "dbeta")
    _check(load_library().gfwa_gate_activation_backward(hpre.data_ptr(), beta.data_ptr(), float(eps),
                                                        dalpha.data_ptr(), dh.data_ptr(), dbeta.data_ptr(),
                                                        B, H, N, _stream()))
    return dh, dbeta


def gfwa_gate_scan_workspace_bytes(B: int, H: int, N: int) -> int:
    return int(load_library().gfwa_gate_scan_workspace_bytes(B, H, N))


def gfwa_gate_prefix_stp(x: torch.Tensor, beta: Optional[torch.Tensor] = None, eps: float = 0.0,
                         c: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """The prefix by scan-then-propagate (for few, very long rows): of x itself when beta is None, else of
    softplus(beta * x) / (beta + eps).  x, beta, c: [B,H,N] fp32 on the GPU."""
    if x.dim() != 3:
        raise ValueError("x must be [B,H,N]")
    B, H, N = x.shape
    _need(x, (B, H, N), torch.float32, "x")
    if beta is not None:
        _need(beta, (B, H, N), torch.float32, "beta")
    if c is None:
        c = torch.empty_like(x)
    _need(c, (B, H, N), torch.float32, "c")
    need = gfwa_gate_scan_workspace_bytes(B, H, N)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=x.device)
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    _check(load_library().gfwa_gate_prefix_stp(x.data_ptr(), beta.data_ptr() if beta is not None else None,
                                               float(eps), c.data_ptr(), workspace.data_ptr(),
                                               workspace.numel() * workspace.element_size(), B, H, N, _stream()))
    return c


def gfwa_forward(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, c: torch.Tensor, w: int,
                 scale: float, O: Optional[torch.Tensor] = None,
                 L: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """O, L of the gated sliding-window attention; Q,K,V: [B,H,N,d], c: [B,H,N] fp32."""
    if Q.dim() != 4:
        raise ValueError("Q must be [B,H,N,d]")
    B, H, N, d = Q.shape
    dt = _dt(Q)
    for name, t in (("Q", Q), ("K", K), ("V", V)):
        _need(t, (B, H, N, d), Q.dtype, name)
    _need(c, (B, H, N), torch.float32, "c")
    if O is None:
        O = torch.empty_like(Q)
    if L is None:
        L = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
    _need(O, (B, H, N, d), Q.dtype, "O")
    _need(L, (B, H, N), torch.float32, "L")
    _check(load_library().gfwa_forward(dt, Q.data_ptr(), K.data_ptr(), V.data_ptr(), c.data_ptr(),
                                       O.data_ptr(), L.data_ptr(), B, H, N, d, int(w), float(scale),
                                       _stream()))
    return O, L


def gfwa_backward_workspace_bytes(dtype: torch.dtype, B: int, H: int, N: int, d: int, w: int) -> int:
    dt = GFWA_BF16 if dtype == torch.bfloat16 else GFWA_F32
    return int(load_library().gfwa_backward_workspace_bytes(dt, B, H, N, d, int(w)))


def gfwa_backward_fast_workspace_bytes(dtype: torch.dtype, B: int, H: int, N: int, d: int, w: int) -> int:
    dt = GFWA_BF16 if dtype == torch.bfloat16 else GFWA_F32
    return int(load_library().gfwa_backward_fast_workspace_bytes(dt, B, H, N, d, int(w)))


def gfwa_backward(Q, K, V, O, dO, c, L, w: int, scale: float, workspace: Optional[torch.Tensor] = None,
                  dQ=None, dK=None, dV=None, dalpha=None):
    """dQ, dK, dV ([B,H,N,d], dtype of Q) and dalpha ([B,H,N] fp32) from the saved O and L.

    workspace: None allocates the minimum; a tensor of gfwa_backward_fast_workspace_bytes selects the
    faster variant of the library (the same holds for gfwa_backward_gqa)."""
    if Q.dim() != 4:
        raise ValueError("Q must be [B,H,N,d]")
    B, H, N, d = Q.shape
    dt = _dt(Q)
    for name, t in (("Q", Q), ("K", K), ("V", V), ("O", O), ("dO", dO)):
        _need(t, (B, H, N, d), Q.dtype, name)
    _need(c, (B, H, N), torch.float32, "c")
    _need(L, (B, H, N), torch.float32, "L")
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(Q) if dK is None else dK
    dV = torch.empty_like(Q) if dV is None else dV
    dalpha = torch.empty((B, H, N), dtype=torch.float32, device=Q.device) if dalpha is None else dalpha
    for name, t in (("dQ", dQ), ("dK", dK), ("dV", dV)):
        _need(t, (B, H, N, d), Q.dtype, name)
    _need(dalpha, (B, H, N), torch.float32, "dalpha")
    need = gfwa_backward_workspace_bytes(Q.dtype, B, H, N, d, w)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(load_library().gfwa_backward(dt, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                        dO.data_ptr(), c.data_ptr(), L.data_ptr(), dQ.data_ptr(),
                                        dK.data_ptr(), dV.data_ptr(), dalpha.data_ptr(),
                                        workspace.data_ptr(), ws_bytes, B, H, N, d, int(w), float(scale),
                                        _stream()))
    return dQ, dK, dV, dalpha


def _kv_heads(Q: torch.Tensor, K: torch.Tensor) -> int:
    if Q.dim() != 4 or K.dim() != 4:
        raise ValueError("Q must be [B,H,N,d] and K [B,Hkv,N,d]")
    H, Hkv = Q.shape[1], K.shape[1]
    if Hkv <= 0 or H % Hkv != 0:
        raise ValueError(f"the number of key/value heads ({Hkv}) must divide the number of query heads ({H})")
    return Hkv


def gfwa_forward_gqa(Q: torch.Tensor, K: torch.Tensor, V: torch.Tensor, c: torch.Tensor, w: int,
                     scale: float, O: Optional[torch.Tensor] = None,
                     L: Optional[torch.Tensor] = None) -> Tuple[torch.Tensor, torch.Tensor]:
    """gfwa_forward with K, V [B,Hkv,N,d]: query head h reads key/value head h // (H // Hkv)."""
    Hkv = _kv_heads(Q, K)
    B, H, N, d = Q.shape
    dt = _dt(Q)
    _need(Q, (B, H, N, d), Q.dtype, "Q")
    for name, t in (("K", K), ("V", V)):
        _need(t, (B, Hkv, N, d), Q.dtype, name)
    _need(c, (B, H, N), torch.float32, "c")
    if O is None:
        O = torch.empty_like(Q)
    if L is None:
        L = torch.empty((B, H, N), dtype=torch.float32, device=Q.device)
    _need(O, (B, H, N, d), Q.dtype, "O")
    _need(L, (B, H, N), torch.float32, "L")
    _check(load_library().gfwa_forward_gqa(dt, Q.data_ptr(), K.data_ptr(), V.data_ptr(), c.data_ptr(),
                                           O.data_ptr(), L.data_ptr(), B, H, Hkv, N, d, int(w), float(scale),
                                           _stream()))
    return O, L


def gfwa_backward_gqa(Q, K, V, O, dO, c, L, w: int, scale: float, workspace: Optional[torch.Tensor] = None,
                      dQ=None, dK=None, dV=None, dalpha=None):
    """gfwa_backward with K, V, dK, dV [B,Hkv,N,d]; dK, dV sum over the query heads of a group."""
    Hkv = _kv_heads(Q, K)
    B, H, N, d = Q.shape
    dt = _dt(Q)
    for name, t in (("Q", Q), ("O", O), ("dO", dO)):
        _need(t, (B, H, N, d), Q.dtype, name)
    for name, t in (("K", K), ("V", V)):
        _need(t, (B, Hkv, N, d), Q.dtype, name)
    _need(c, (B, H, N), torch.float32, "c")
    _need(L, (B, H, N), torch.float32, "L")
    dQ = torch.empty_like(Q) if dQ is None else dQ
    dK = torch.empty_like(K) if dK is None else dK
    dV = torch.empty_like(K) if dV is None else dV
    dalpha = torch.empty((B, H, N), dtype=torch.float32, device=Q.device) if dalpha is None else dalpha
    _need(dQ, (B, H, N, d), Q.dtype, "dQ")
    for name, t in (("dK", dK), ("dV", dV)):
        _need(t, (B, Hkv, N, d), Q.dtype, name)
    _need(dalpha, (B, H, N), torch.float32, "dalpha")
    need = gfwa_backward_workspace_bytes(Q.dtype, B, H, N, d, w)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=Q.device)
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    ws_bytes = workspace.numel() * workspace.element_size()
    _check(load_library().gfwa_backward_gqa(dt, Q.data_ptr(), K.data_ptr(), V.data_ptr(), O.data_ptr(),
                                            dO.data_ptr(), c.data_ptr(), L.data_ptr(), dQ.data_ptr(),
                                            dK.data_ptr(), dV.data_ptr(), dalpha.data_ptr(),
                                            workspace.data_ptr(), ws_bytes, B, H, Hkv, N, d, int(w),
                                            float(scale), _stream()))
    return dQ, dK, dV, dalpha


def gfwa_decode_workspace_bytes(B: int, H: int, T: int, d: int, w: int) -> int:
    return int(load_library().gfwa_decode_workspace_bytes(B, H, T, d, int(w)))


def gfwa_decode(q: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor, c: torch.Tensor, pos: torch.Tensor, w: int,
                scale: float, alpha_t: Optional[torch.Tensor] = None, o: Optional[torch.Tensor] = None,
                L: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None):
    """One decoding step: q [B,H,d] against the caches Kc, Vc [B,Hkv,T,d] at positions pos [B] (int32);
    c [B,H,T] fp32 (entry pos is written when alpha_t [B,H] is given).  Returns o [B,H,d], L [B,H]."""
    if q.dim() != 3 or Kc.dim() != 4:
        raise ValueError("q must be [B,H,d] and Kc [B,Hkv,T,d]")
    B, H, d = q.shape
    Hkv, T = Kc.shape[1], Kc.shape[2]
    if Hkv <= 0 or H % Hkv != 0:
        raise ValueError(f"the number of key/value heads ({Hkv}) must divide the number of query heads ({H})")
    dt = _dt(q)
    _need(q, (B, H, d), q.dtype, "q")
    for name, t in (("Kc", Kc), ("Vc", Vc)):
        _need(t, (B, Hkv, T, d), q.dtype, name)
    _need(c, (B, H, T), torch.float32, "c")
    _need(pos, (B,), torch.int32, "pos")
    if alpha_t is not None:
        _need(alpha_t, (B, H), torch.float32, "alpha_t")
    if o is None:
        o = torch.empty_like(q)
    if L is None:
        L = torch.empty((B, H), dtype=torch.float32, device=q.device)
    _need(o, (B, H, d), q.dtype, "o")
    _need(L, (B, H), torch.float32, "L")
    need = gfwa_decode_workspace_bytes(B, H, T, d, w)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    if not workspace.is_cuda or not workspace.is_contiguous():
        raise ValueError("workspace must be a contiguous GPU tensor")
    _check(load_library().gfwa_decode(dt, q.data_ptr(), Kc.data_ptr(), Vc.data_ptr(), c.data_ptr(),
                                      alpha_t.data_ptr() if alpha_t is not None else None, pos.data_ptr(),
                                      o.data_ptr(), L.data_ptr(), workspace.data_ptr(),
                                      workspace.numel() * workspace.element_size(), B, H, Hkv, T, d, int(w),
                                      float(scale), _stream()))
    return o, L


def gfwa_decode_static(q: torch.Tensor, Kc: torch.Tensor, Vc: torch.Tensor, c: torch.Tensor, pos: torch.Tensor,
                       w: int, scale: float, o: torch.Tensor, L: torch.Tensor,
                       alpha_t: Optional[torch.Tensor] = None):
    """gfwa_decode without a workspace and without any allocation: the caller passes the outputs
    o [B,H,d] and L [B,H]; the partial results live in the library's own scratch."""
    if q.dim() != 3 or Kc.dim() != 4:
        raise ValueError("q must be [B,H,d] and Kc [B,Hkv,T,d]")
    B, H, d = q.shape
    Hkv, T = Kc.shape[1], Kc.shape[2]
    if Hkv <= 0 or H % Hkv != 0:
        raise ValueError(f"the number of key/value heads ({Hkv}) must divide the number of query heads ({H})")
    dt = _dt(q)
    _need(q, (B, H, d), q.dtype, "q")
    for name, t in (("Kc", Kc), ("Vc", Vc)):
        _need(t, (B, Hkv, T, d), q.dtype, name)
    _need(c, (B, H, T), torch.float32, "c")
    _need(pos, (B,), torch.int32, "pos")
    if alpha_t is not None:
        _need(alpha_t, (B, H), torch.float32, "alpha_t")
    _need(o, (B, H, d), q.dtype, "o")
    _need(L, (B, H), torch.float32, "L")
    _check(load_library().gfwa_decode_static(dt, q.data_ptr(), Kc.data_ptr(), Vc.data_ptr(), c.data_ptr(),
                                             alpha_t.data_ptr() if alpha_t is not None else None, pos.data_ptr(),
                                             o.data_ptr(), L.data_ptr(), B, H, Hkv, T, d, int(w), float(scale),
                                             _stream()))
    return o, L


def gfwa_probe_mfma(sink: torch.Tensor, iterations: int, workgroups: int, random_operands: int = 0) -> float:
    """Enqueue the bf16 MFMA loop (0: constant operands, 1: pseudo-random operands, 2: pseudo-random operands
    plus one LDS fragment read and five vector instructions per MFMA); returns the floating-point operations
    of the launch."""
    _need(sink, tuple(sink.shape), torch.float32, "sink")
    flops = ctypes.c_double(0.0)
    _check(load_library().gfwa_probe_mfma(sink.data_ptr(), int(iterations), int(workgroups), int(random_operands),
                                          ctypes.byref(flops),
                                          _stream()))
    return float(flops.value)


def gfwa_probe_copy(src: torch.Tensor, dst: torch.Tensor) -> int:
    """Enqueue a plain copy of src into dst (same size, contiguous); returns the bytes copied."""
    if not (src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()):
        raise ValueError("src and dst must be contiguous GPU tensors")
    nbytes = src.numel() * src.element_size()
    if nbytes != dst.numel() * dst.element_size():
        raise ValueError("src and dst differ in size")
    _check(load_library().gfwa_probe_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream()))
    return nbytes


def gfwa_profile_enable(on: bool) -> None:
    """Start (clearing old records) or stop per-kernel HIP-event timing inside the library."""
    _check(load_library().gfwa_profile_enable(1 if on else 0))


def gfwa_profile_read() -> dict:
    """{kernel name: (total ms, launches)} for the launches recorded since profiling was enabled."""
    ms = (ctypes.c_float * N_KERNELS)()
    cnt = (ctypes.c_int * N_KERNELS)()
    _check(load_library().gfwa_profile_read(ms, cnt, N_KERNELS))
    return {gfwa_profile_kernel_name(k): (float(ms[k]), int(cnt[k])) for k in range(N_KERNELS)}


def gfwa_profile_kernel_name(k: int) -> str:
    return load_library().gfwa_profile_kernel_name(int(k)).decode()
