"""Seeded synthetic workloads shared by the tests, the benchmark and the oracle checks.

This module only draws numbers and shapes.  It holds none of the method's
arithmetic (no scores, no sigmoid, no gradients) and imports neither the HIP
binding nor the oracle, so both sides can be fed from it.

The five named workloads follow the benchmark configurations of this build; they
stand in for batches of single-cell gene-token sequences (paper Sec. 1 / Sec. 5.1:
jagged per-cell lengths, right-padded to the batch maximum; 160M-model head
shape H=12, d=64 from the architecture table), which are not available offline.

Recipe (numpy ``default_rng(seed)``, in this order): valid lengths first, then
Q, K, V, dO as float32 normal draws over the WHOLE padded tensor (padded rows
hold finite random data on purpose), each rounded to bf16 with
round-to-nearest-even.  ``scale = 1/sqrt(d)``, ``bias[z] = -ln(n_z)`` (the
paper's b = -log n with n the sequence's valid length; 0 for an empty sequence).
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field
from typing import Dict, Optional, Sequence

import numpy as np

WORKLOADS: Dict[str, dict] = {
    # name: B, H, d, N_max, length rule, std of Q/K/V, std of dO
    "tiny": dict(B=2, H=2, d=64, N=256, lengths=("fixed", (256, 173)), qkv_std=1.0, do_std=1.0),
    "unpadded": dict(B=8, H=12, d=64, N=2048, lengths=("full",), qkv_std=1.0, do_std=1.0),
    "jagged": dict(B=16, H=12, d=64, N=4096, lengths=("lognormal", 1500.0, 0.8, 64, 4096), qkv_std=1.0, do_std=1.0),
    "long": dict(B=4, H=12, d=64, N=8192, lengths=("uniform", 1024, 8192), qkv_std=math.sqrt(2.0), do_std=1.0),
    "long_full": dict(B=4, H=12, d=64, N=8192, lengths=("full",), qkv_std=math.sqrt(2.0), do_std=1.0),
    "wide": dict(B=2, H=16, d=128, N=16384, lengths=("uniform", 12000, 16384), qkv_std=1.0, do_std=1.0),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even); result stays float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of float32 values that are already bf16-representable."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    if np.any(u & 0xFFFF):
        raise ValueError("values are not bf16-representable")
    return (u >> 16).astype(np.uint16).reshape(x.shape)


def bits_to_f32(b: np.ndarray) -> np.ndarray:
    """float32 values of bf16 bit patterns (uint16 or int16 storage)."""
    b = np.ascontiguousarray(b).view(np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32).reshape(b.shape)


def draw_lengths(rule: Sequence, B: int, N: int, rng: np.random.Generator) -> np.ndarray:
    kind = rule[0]
    if kind == "fixed":
        n = np.asarray(rule[1], dtype=np.int64)
        if n.shape != (B,):
            raise ValueError("fixed lengths must have B entries")
    elif kind == "full":
        n = np.full(B, N, dtype=np.int64)
    elif kind == "lognormal":
        _, median, sigma, lo, hi = rule
        n = np.rint(np.exp(math.log(median) + sigma * rng.standard_normal(B))).astype(np.int64)
        n = np.clip(n, lo, hi)
    elif kind == "uniform":
        _, lo, hi = rule
        n = rng.integers(lo, hi + 1, size=B, dtype=np.int64)
    else:
        raise ValueError(f"unknown length rule {kind!r}")
    return np.clip(n, 0, N).astype(np.int32)


@dataclass
class Workload:
    name: str
    seed: int
    B: int
    N: int
    H: int
    d: int
    scale: float
    seqlens: np.ndarray  # int32 [B]
    bias: np.ndarray     # float32 [B]
    q: np.ndarray        # float32 [B, N, H, d], bf16-representable
    k: np.ndarray
    v: np.ndarray
    d_o: np.ndarray
    meta: dict = field(default_factory=dict)

    def bits(self, which: str) -> np.ndarray:
        return bf16_bits(getattr(self, which))


def default_bias(seqlens: np.ndarray) -> np.ndarray:
    n = np.maximum(np.asarray(seqlens, dtype=np.float64), 1.0)
    return (-np.log(n)).astype(np.float32)


def make(B: int, N: int, H: int, d: int, seqlens: Sequence[int], seed: int = 0, qkv_std: float = 1.0,
         do_std: float = 1.0, bias: Optional[Sequence[float]] = None, scale: Optional[float] = None,
         name: str = "custom", rng: Optional[np.random.Generator] = None) -> Workload:
    """A workload with explicit shape and valid lengths (used for edge-case tests)."""
    if rng is None:
        rng = np.random.default_rng(seed)
    seqlens = np.asarray(seqlens, dtype=np.int32)
    if seqlens.shape != (B,):
        raise ValueError("seqlens must have B entries")
    shape = (B, N, H, d)

    def draw(std: float) -> np.ndarray:
        x = rng.standard_normal(shape, dtype=np.float32)
        if std != 1.0:
            x *= np.float32(std)
        return round_to_bf16(x)

    q = draw(qkv_std)
    k = draw(qkv_std)
    v = draw(qkv_std)
    d_o = draw(do_std)
    b = default_bias(seqlens) if bias is None else np.asarray(bias, dtype=np.float32)
    s = 1.0 / math.sqrt(d) if scale is None else float(scale)
    return Workload(name=name, seed=seed, B=B, N=N, H=H, d=d, scale=s, seqlens=seqlens, bias=b,
                    q=q, k=k, v=v, d_o=d_o,
                    meta=dict(qkv_std=qkv_std, do_std=do_std, lengths=[int(x) for x in seqlens]))


def generate(name: str, seed: int = 0) -> Workload:
    """One of the named workloads, fully determined by (name, seed)."""
    cfg = WORKLOADS[name]
    rng = np.random.default_rng(seed)
    seqlens = draw_lengths(cfg["lengths"], cfg["B"], cfg["N"], rng)
    return make(cfg["B"], cfg["N"], cfg["H"], cfg["d"], seqlens, seed=seed, qkv_std=cfg["qkv_std"],
                do_std=cfg["do_std"], name=name, rng=rng)
