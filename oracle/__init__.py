"""GatedFWA CPU oracle (fp64) -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.

Thin ctypes layer over `gfwa_oracle.c` plus loops over (batch, head).  Only the
tests, `__graft_entry__.smoke()` and the `cpu_baseline` leg of `bench.py` may
import this package; the HIP path never does, and this package never imports
the HIP path.

All functions take and return numpy arrays; floating inputs are upcast to fp64
exactly.  Shapes follow the problem statement of Alg. 2 / Alg. 3 of the paper
with a leading [B, H]: Q, K, V, O, dO, dQ, dK, dV are [B,H,N,d]; alpha, c, L,
dalpha are [B,H,N].
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gfwa_oracle.c")
# GFWA_ORACLE_LIB names another build of gfwa_oracle.c (a sanitizer build, for one); it is loaded as it is
_LIB = os.environ.get("GFWA_ORACLE_LIB") or os.path.join(_HERE, "libgfwa_oracle.so")
_lib: Optional[ctypes.CDLL] = None

_dp = ctypes.POINTER(ctypes.c_double)


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (fp64, OpenMP, no fast-math)."""
    if os.environ.get("GFWA_ORACLE_LIB"):
        return _LIB
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        L = ctypes.c_long
        D = ctypes.c_double
        lib.gfwa_oracle_threads.restype = ctypes.c_int
        lib.gfwa_oracle_prefix.argtypes = [_dp, _dp, L]
        lib.gfwa_oracle_forward_c.argtypes = [_dp, _dp, _dp, _dp, L, L, L, D, _dp, _dp, _dp]
        lib.gfwa_oracle_forward.argtypes = [_dp, _dp, _dp, _dp, L, L, L, D, _dp, _dp, _dp]
        lib.gfwa_oracle_backward_c.argtypes = [_dp, _dp, _dp, _dp, _dp, L, L, L, D,
                                               _dp, _dp, _dp, _dp, _dp]
        lib.gfwa_oracle_backward_saved_O.argtypes = [_dp, _dp, _dp, _dp, _dp, _dp, L, L, L, D,
                                                     _dp, _dp, _dp, _dp, _dp]
        lib.gfwa_oracle_dalpha_from_dc.argtypes = [_dp, _dp, L]
        lib.gfwa_oracle_dalpha_direct.argtypes = [_dp, _dp, L, L]
        lib.gfwa_oracle_gate_activation.argtypes = [_dp, _dp, D, _dp, L]
        lib.gfwa_oracle_gate_activation_backward.argtypes = [_dp, _dp, D, _dp, _dp, _dp, L]
        for f in ("gfwa_oracle_prefix", "gfwa_oracle_forward_c", "gfwa_oracle_forward",
                  "gfwa_oracle_backward_c", "gfwa_oracle_backward_saved_O", "gfwa_oracle_dalpha_from_dc",
                  "gfwa_oracle_dalpha_direct", "gfwa_oracle_gate_activation",
                  "gfwa_oracle_gate_activation_backward"):
            getattr(lib, f).restype = None
        _lib = lib
    return _lib


def threads() -> int:
    """Number of host threads the oracle's OpenMP loops use."""
    return int(_load().gfwa_oracle_threads())


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x), dtype=np.float64)


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(_dp)


def _flat_heads(x: np.ndarray, trailing: int) -> np.ndarray:
    """[..., N(, d)] -> [BH, N(, d)] view."""
    x = _f64(x)
    return x.reshape((-1,) + x.shape[-trailing:])


# --------------------------------------------------------------------------
# gate prefix (Sec. 3.2)
# --------------------------------------------------------------------------
def gate_prefix(alpha) -> np.ndarray:
    """c[..., t] = sum_{q<=t} alpha[..., q], fp64."""
    lib = _load()
    a = _flat_heads(alpha, 1)
    c = np.empty_like(a)
    for r in range(a.shape[0]):
        lib.gfwa_oracle_prefix(_p(a[r]), _p(c[r]), a.shape[1])
    return c.reshape(np.shape(alpha))


# --------------------------------------------------------------------------
# forward (Sec. 3.2 score, Alg. 2 outputs)
# --------------------------------------------------------------------------
def gate_activation(h, beta, eps: float) -> np.ndarray:
    """alpha = softplus(beta * h) / (beta + eps), elementwise (Sec. 3.2; Alg. 1 on-chip steps)."""
    h, beta = _f64(h), _f64(beta)
    assert h.shape == beta.shape
    alpha = np.empty_like(h)
    _load().gfwa_oracle_gate_activation(_p(h), _p(beta), float(eps), _p(alpha), h.size)
    return alpha


def gate_activation_backward(h, beta, eps: float, dalpha):
    """(dh, dbeta) for a given d(alpha): the chain rule on the definition of the gate."""
    h, beta, dalpha = _f64(h), _f64(beta), _f64(dalpha)
    assert h.shape == beta.shape == dalpha.shape
    dh, dbeta = np.empty_like(h), np.empty_like(h)
    _load().gfwa_oracle_gate_activation_backward(_p(h), _p(beta), float(eps), _p(dalpha), _p(dh), _p(dbeta), h.size)
    return dh, dbeta


def forward_from_c(Q, K, V, c, w: int, scale: float, return_P: bool = False):
    """O, L (and optionally the band of P as [.., N, min(w,N)]) from a given prefix c."""
    lib = _load()
    Qf, Kf, Vf = (_flat_heads(x, 2) for x in (Q, K, V))
    cf = _flat_heads(c, 1)
    BH, N, d = Qf.shape
    O = np.empty_like(Qf)
    L = np.empty((BH, N), dtype=np.float64)
    wb = min(int(w), N)
    P = np.empty((BH, N, wb), dtype=np.float64) if return_P else None
    for r in range(BH):
        lib.gfwa_oracle_forward_c(_p(Qf[r]), _p(Kf[r]), _p(Vf[r]), _p(cf[r]), N, d, int(w),
                                  float(scale), _p(O[r]), _p(L[r]),
                                  _p(P[r]) if return_P else None)
    O = O.reshape(np.shape(Q))
    L = L.reshape(np.shape(c))
    if return_P:
        return O, L, P.reshape(np.shape(c) + (wb,))
    return O, L


def forward(Q, K, V, alpha, w: int, scale: float):
    """The full definition: prefix in fp64, then the gated windowed softmax.  Returns O, L, c."""
    c = gate_prefix(alpha)
    O, L = forward_from_c(Q, K, V, c, w, scale)
    return O, L, c


# --------------------------------------------------------------------------
# backward (App. E.2, Alg. 3)
# --------------------------------------------------------------------------
def backward_from_c(Q, K, V, c, dO, w: int, scale: float, return_dS: bool = False,
                    O_saved=None) -> Dict[str, np.ndarray]:
    """dQ, dK, dV, dc (gradient w.r.t. the prefix) and dalpha (reverse inclusive scan of dc).
    With O_saved [.., N, d]: Alg. 3 evaluated on that saved forward output (D = rowsum(dO * O_saved))
    instead of on the exact output - what the algorithm returns when O was rounded for storage."""
    lib = _load()
    Qf, Kf, Vf, dOf = (_flat_heads(x, 2) for x in (Q, K, V, dO))
    Of = None if O_saved is None else _flat_heads(O_saved, 2)
    assert Of is None or Of.shape == Qf.shape
    cf = _flat_heads(c, 1)
    BH, N, d = Qf.shape
    wb = min(int(w), N)
    dQ, dK, dV = np.empty_like(Qf), np.empty_like(Qf), np.empty_like(Qf)
    dc = np.empty((BH, N), dtype=np.float64)
    dalpha = np.empty((BH, N), dtype=np.float64)
    dS = np.empty((BH, N, wb), dtype=np.float64) if return_dS else None
    for r in range(BH):
        if Of is None:
            lib.gfwa_oracle_backward_c(_p(Qf[r]), _p(Kf[r]), _p(Vf[r]), _p(cf[r]), _p(dOf[r]), N, d,
                                       int(w), float(scale), _p(dQ[r]), _p(dK[r]), _p(dV[r]),
                                       _p(dc[r]), _p(dS[r]) if return_dS else None)
        else:
            lib.gfwa_oracle_backward_saved_O(_p(Qf[r]), _p(Kf[r]), _p(Vf[r]), _p(cf[r]), _p(dOf[r]), _p(Of[r]),
                                             N, d, int(w), float(scale), _p(dQ[r]), _p(dK[r]), _p(dV[r]),
                                             _p(dc[r]), _p(dS[r]) if return_dS else None)
        lib.gfwa_oracle_dalpha_from_dc(_p(dc[r]), _p(dalpha[r]), N)
    shp, vshp = np.shape(Q), np.shape(c)
    out = {"dQ": dQ.reshape(shp), "dK": dK.reshape(shp), "dV": dV.reshape(shp),
           "dc": dc.reshape(vshp), "dalpha": dalpha.reshape(vshp)}
    if return_dS:
        out["dS"] = dS.reshape(vshp + (wb,))
    return out


def backward(Q, K, V, alpha, dO, w: int, scale: float, return_dS: bool = False) -> Dict[str, np.ndarray]:
    return backward_from_c(Q, K, V, gate_prefix(alpha), dO, w, scale, return_dS=return_dS)


# --------------------------------------------------------------------------
# grouped-query layout (App. "Additional Experiment Details": heads_per_gqa_group in the training
# tables).  The paper fixes only the group size; the reading taken is the usual one: query head h
# attends to the keys and values of head h // G, the gate belongs to the query head.  The definition
# written out: repeat each key/value head G times, apply the multi-head definition, and sum the
# key/value gradients over the G query heads that read the same head.
# --------------------------------------------------------------------------
def _repeat_kv(X, H: int) -> np.ndarray:
    X = _f64(X)
    B, Hkv = X.shape[0], X.shape[1]
    assert X.ndim == 4 and H % Hkv == 0, "K, V must be [B,Hkv,N,d] with Hkv dividing H"
    return np.repeat(X, H // Hkv, axis=1)


def forward_gqa_from_c(Q, K, V, c, w: int, scale: float):
    """O, L for Q [B,H,N,d], K, V [B,Hkv,N,d], c [B,H,N]."""
    H = np.shape(Q)[1]
    return forward_from_c(Q, _repeat_kv(K, H), _repeat_kv(V, H), c, w, scale)


def backward_gqa_from_c(Q, K, V, c, dO, w: int, scale: float, O_saved=None) -> Dict[str, np.ndarray]:
    """dQ [B,H,N,d], dK, dV [B,Hkv,N,d], dc, dalpha [B,H,N]."""
    B, H, N, d = np.shape(Q)
    Hkv = np.shape(K)[1]
    out = backward_from_c(Q, _repeat_kv(K, H), _repeat_kv(V, H), c, dO, w, scale, O_saved=O_saved)
    for k in ("dK", "dV"):
        out[k] = out[k].reshape(B, Hkv, H // Hkv, N, d).sum(axis=2)
    return out


# --------------------------------------------------------------------------
# decoding step with a key/value cache (Sec. 1: O(wd) work per generated token).  It is row `pos` of
# the forward definition, written out directly: one query per (b, h) against the cached keys and
# values of positions max(0, pos-w+1) .. pos.
# --------------------------------------------------------------------------
def decode_from_c(q, Kc, Vc, c, pos, w: int, scale: float):
    """o [B,H,d], L [B,H] for q [B,H,d], caches Kc, Vc [B,Hkv,T,d], prefix c [B,H,T] (c[..., pos] included)
    and the current position pos[b] of every batch entry."""
    q, Kc, Vc, c = _f64(q), _f64(Kc), _f64(Vc), _f64(c)
    B, H, d = q.shape
    Hkv = Kc.shape[1]
    assert H % Hkv == 0 and c.shape[:2] == (B, H) and c.shape[2] == Kc.shape[2]
    G = H // Hkv
    o = np.empty((B, H, d))
    L = np.empty((B, H))
    for b in range(B):
        p = int(pos[b])
        lo = max(0, p - int(w) + 1)
        for h in range(H):
            K = Kc[b, h // G, lo:p + 1]
            V = Vc[b, h // G, lo:p + 1]
            s = scale * (K @ q[b, h]) + (c[b, h, lo:p + 1] - c[b, h, p])
            m = s.max()
            e = np.exp(s - m)
            L[b, h] = m + np.log(e.sum())
            o[b, h] = (e / e.sum()) @ V
    return o, L


def dalpha_direct(dS_band, w: int) -> np.ndarray:
    """d(alpha) from the band of dS without going through dc (tiny N only)."""
    lib = _load()
    dSf = _flat_heads(dS_band, 2)
    BH, N, _ = dSf.shape
    out = np.empty((BH, N), dtype=np.float64)
    for r in range(BH):
        lib.gfwa_oracle_dalpha_direct(_p(dSf[r]), _p(out[r]), N, int(w))
    return out.reshape(np.shape(dS_band)[:-1])


def select_heads(x: np.ndarray, heads: Sequence[int], trailing: int) -> np.ndarray:
    """Rows `heads` of the flattened [B*H, ...] view (for parity on a sample of heads)."""
    flat = np.asarray(x).reshape((-1,) + np.shape(x)[-trailing:])
    return np.ascontiguousarray(flat[np.asarray(heads)])
