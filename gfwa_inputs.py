"""Seeded synthetic inputs for GatedFWA (gated sliding-window attention).

This module serves both the CPU oracle and the HIP path and therefore holds
none of the method's arithmetic: it only draws random tensors of the shapes and
value distributions of the paper's language-modelling workloads (Sec. 5,
App. F: N=4096/w=512 with 64-wide heads; kernel benchmark w in {512,1024},
long N) and rounds them to the storage type.

Every tensor is returned as a float32 numpy array whose values are exactly
representable in the workload's storage type (bf16 or fp32), so that
`x.astype(np.float64)` (oracle) and `torch.from_numpy(x).to(torch.bfloat16)`
(device) see bit-identical numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

SEED_BASE = 0x251207782000
TAG = {"Q": 0, "K": 1, "V": 2, "alpha": 3, "dO": 4}


# --------------------------------------------------------------------------
# storage-format helpers (bit manipulation only)
# --------------------------------------------------------------------------
def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> 16).astype(np.uint16).reshape(x.shape)


def bf16_ulp(x: np.ndarray) -> np.ndarray:
    """Spacing of bf16 numbers at |x| (8 significand bits)."""
    ax = np.maximum(np.abs(np.asarray(x, dtype=np.float64)), 2.0 ** -126)
    return 2.0 ** (np.floor(np.log2(ax)) - 7)


# --------------------------------------------------------------------------
# random draws
# --------------------------------------------------------------------------
def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=seed))


def normal(seed: int, shape, mean: float = 0.0, std: float = 1.0) -> np.ndarray:
    """fp64 N(mean, std^2) draws from a counter-based generator keyed by `seed`."""
    return _rng(seed).standard_normal(size=shape) * std + mean


def softplus(z: np.ndarray) -> np.ndarray:
    """log(1+e^z) in fp64 (input recipe for the non-negative gate alpha)."""
    z = np.asarray(z, dtype=np.float64)
    return np.maximum(z, 0.0) + np.log1p(np.exp(-np.abs(z)))


# --------------------------------------------------------------------------
# workloads
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    index: int                 # enters the seed
    B: int
    H: int
    N: int
    d: int
    w: int
    dtype: str                 # "bf16" or "f32": storage type of Q,K,V,O,dO
    qkv_std: float = 1.0
    alpha_mu: float = 0.0      # alpha = softplus(N(alpha_mu, 1))
    zero_gate_heads: Tuple[int, ...] = ()   # heads whose alpha is exactly 0
    backward: bool = False
    kv_heads: int = 0          # key/value heads of the grouped-query layout; 0: one per query head

    @property
    def Hkv(self) -> int:
        return self.kv_heads or self.H

    @property
    def scale(self) -> float:
        return 1.0 / float(np.sqrt(self.d))

    def seed(self, tag: str) -> int:
        return SEED_BASE + 16 * self.index + TAG[tag]

    # FLOP conventions of the metric: only in-window pairs are counted.
    def flops_fwd_nominal(self) -> float:
        return 4.0 * self.B * self.H * self.N * self.w * self.d

    def flops_fwd_exact(self) -> float:
        wp = min(self.w, self.N)
        pairs = self.N * wp - wp * (wp - 1) // 2
        return 4.0 * self.B * self.H * self.d * pairs

    def flops_bwd_nominal(self) -> float:
        return 10.0 * self.B * self.H * self.N * self.w * self.d


WORKLOADS: Dict[str, Workload] = {
    wl.name: wl
    for wl in [
        Workload("tiny_fwd_f32", 0, 1, 1, 256, 64, 64, "f32", alpha_mu=0.0),
        Workload("lm_fwd", 1, 4, 16, 4096, 64, 512, "bf16", alpha_mu=-2.0),
        Workload("long_fwd", 2, 1, 32, 16384, 128, 1024, "bf16", alpha_mu=-3.0),
        Workload("gate_extreme_fwd", 3, 2, 8, 8192, 128, 2048, "bf16", qkv_std=3.0,
                 alpha_mu=1.0, zero_gate_heads=(0, 1, 2, 3)),
        Workload("train_bwd", 4, 4, 16, 8192, 128, 1024, "bf16", alpha_mu=-2.0, backward=True),
        Workload("long_bwd", 5, 1, 32, 16384, 128, 1024, "bf16", alpha_mu=-3.0, backward=True),
        # grouped-query variants, 4 query heads per key/value head as in the paper's training tables
        Workload("lm_gqa_bwd", 6, 4, 16, 4096, 64, 512, "bf16", alpha_mu=-2.0, backward=True, kv_heads=4),
        Workload("long_gqa_bwd", 7, 1, 32, 16384, 128, 1024, "bf16", alpha_mu=-3.0, backward=True, kv_heads=8),
        # fp32 storage at a size that fills the chip (the fp32 matrix-core kernels)
        Workload("mid_bwd_f32", 8, 2, 16, 4096, 128, 1024, "f32", alpha_mu=-2.0, backward=True),
    ]
}


def custom(name: str, B: int, H: int, N: int, d: int, w: int, dtype: str = "bf16", index: int = 15,
           **kw) -> Workload:
    """A workload outside the named list (tests: ragged sizes, tiny shapes)."""
    return Workload(name, index, B, H, N, d, w, dtype, **kw)


def _store(x: np.ndarray, dtype: str) -> np.ndarray:
    x32 = x.astype(np.float32)
    return round_to_bf16(x32) if dtype == "bf16" else x32


def make_tensor(wl: Workload, tag: str, heads: Optional[np.ndarray] = None) -> np.ndarray:
    """One tensor of the workload; `heads` (flat b*H+h indices) restricts the result to
    those rows of the [B*H, ...] view but draws exactly the same numbers."""
    BH = wl.B * wl.H
    if tag == "alpha":
        z = normal(wl.seed(tag), (BH, wl.N), mean=wl.alpha_mu)
        a = softplus(z).astype(np.float32)
        for h in wl.zero_gate_heads:
            a.reshape(wl.B, wl.H, wl.N)[:, h, :] = 0.0
        out = a
    else:
        std = wl.qkv_std if tag in ("Q", "K", "V") else 1.0
        if tag in ("K", "V"):
            BH = wl.B * wl.Hkv
        out = _store(normal(wl.seed(tag), (BH, wl.N, wl.d), std=std), wl.dtype)
    if heads is not None:
        return np.ascontiguousarray(out[np.asarray(heads)])
    return out.reshape((wl.B, BH // wl.B) + out.shape[1:])


def make_gate_inputs(wl: Workload) -> Tuple[np.ndarray, np.ndarray]:
    """Inputs of the gate activation, [B,H,N] fp32: the pre-activation h ~ N(alpha_mu, 1) (the same draw
    that `alpha` is the softplus of) and a positive amplitude beta, log-normal with median 1."""
    shape = (wl.B, wl.H, wl.N)
    h = normal(wl.seed("alpha"), (wl.B * wl.H, wl.N), mean=wl.alpha_mu).reshape(shape).astype(np.float32)
    beta = np.exp(0.5 * normal(wl.seed("alpha") + 1000003, shape)).astype(np.float32)
    return h, beta


def make_inputs(wl: Workload) -> Dict[str, np.ndarray]:
    """All input tensors: Q,K,V [B,H,N,d], alpha [B,H,N] (fp32, >= 0), and dO for backward."""
    tags = ["Q", "K", "V", "alpha"] + (["dO"] if wl.backward else [])
    return {t: make_tensor(wl, t) for t in tags}
