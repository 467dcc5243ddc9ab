"""Python face of the fp64 oracle -- TEST INFRASTRUCTURE ONLY (see the C file's header).

Two independent evaluators of the same definition (paper Sec. 3, sigmoid-attention
equation; appendix Alg. 1-3 for padding and gradients):

* ``fwd`` / ``bwd`` / ``matrices`` call the plain-C triple loops in
  ``sigmoid_attn_oracle.c`` (whole (z, h) slices, every row);
* ``fwd_rows`` / ``bwd_q_rows`` / ``bwd_kv_rows`` evaluate single output rows with
  numpy fp64 matrix-vector products, so that sampled outputs of a full-size
  workload can be checked one by one.

All tensors are ``[B, N, H, d]`` float32 numpy arrays holding bf16-representable
values (widened exactly to fp64); ``seqlens`` is int32 ``[B]`` (valid prefix
length per sequence), ``bias`` is ``[B]``.  Outputs are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Iterable, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "sigmoid_attn_oracle.c")
_LIB = os.path.join(_HERE, "libsigattn_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    """Compile the C oracle with gcc (x86-64-v3 so the binary also runs on other hosts)."""
    if force or not os.path.exists(_LIB):
        cmd = ["gcc", "-O3", "-march=x86-64-v3", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_F = ctypes.POINTER(ctypes.c_float)
_D = ctypes.POINTER(ctypes.c_double)
_I = ctypes.POINTER(ctypes.c_int32)


def _load():
    global _lib
    if _lib is None:
        build(force=False)
        lib = ctypes.CDLL(_LIB)
        ci, cd = ctypes.c_int, ctypes.c_double
        lib.sigattn_oracle_threads.restype = ci
        lib.sigattn_oracle_fwd_slice.argtypes = [_F, _F, _F, _D, _I, _D, cd, ci, ci, ci, ci, ci, ci]
        lib.sigattn_oracle_fwd_slice.restype = None
        lib.sigattn_oracle_bwd_slice.argtypes = [_F, _F, _F, _F, _D, _D, _D, _I, _D, cd, ci, ci, ci, ci, ci, ci]
        lib.sigattn_oracle_bwd_slice.restype = None
        lib.sigattn_oracle_fwd.argtypes = [_F, _F, _F, _D, _I, _D, cd, ci, ci, ci, ci]
        lib.sigattn_oracle_fwd.restype = None
        lib.sigattn_oracle_bwd.argtypes = [_F, _F, _F, _F, _D, _D, _D, _I, _D, cd, ci, ci, ci, ci]
        lib.sigattn_oracle_bwd.restype = None
        lib.sigattn_oracle_matrices.argtypes = [_F, _F, _F, _F, _D, _D, _D, _I, _D, cd, ci, ci, ci, ci, ci, ci]
        lib.sigattn_oracle_matrices.restype = None
        lib.sigattn_oracle_cross_fwd.argtypes = [_F, _F, _F, _D, _I, _I, _D, cd, ci, ci, ci, ci, ci]
        lib.sigattn_oracle_cross_fwd.restype = None
        lib.sigattn_oracle_cross_bwd.argtypes = [_F, _F, _F, _F, _D, _D, _D, _D, _I, _I, _D, cd, ci, ci, ci, ci, ci]
        lib.sigattn_oracle_cross_bwd.restype = None
        _lib = lib
    return _lib


def threads() -> int:
    """Number of OpenMP threads the C oracle will use."""
    return int(_load().sigattn_oracle_threads())


def _f32(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.ndim != 4:
        raise ValueError("expected a [B, N, H, d] array")
    return a


def _common(q, k, v, seqlens, bias):
    q, k, v = _f32(q), _f32(k), _f32(v)
    if not (q.shape == k.shape == v.shape):
        raise ValueError("q, k, v must share one shape")
    B, N, H, d = q.shape
    seqlens = np.ascontiguousarray(seqlens, dtype=np.int32)
    bias = np.ascontiguousarray(bias, dtype=np.float64)
    if seqlens.shape != (B,) or bias.shape != (B,):
        raise ValueError("seqlens and bias must have shape [B]")
    return q, k, v, seqlens, bias, (B, N, H, d)


def _p(a, t):
    return a.ctypes.data_as(t)


def fwd(q, k, v, seqlens, bias, scale: float,
        slices: Optional[Iterable[Tuple[int, int]]] = None) -> np.ndarray:
    """O for every (z, h) slice, or only for the listed ones (others stay 0)."""
    q, k, v, seqlens, bias, (B, N, H, d) = _common(q, k, v, seqlens, bias)
    lib = _load()
    o = np.zeros((B, N, H, d), dtype=np.float64)
    if slices is None:
        lib.sigattn_oracle_fwd(_p(q, _F), _p(k, _F), _p(v, _F), _p(o, _D), _p(seqlens, _I), _p(bias, _D),
                               float(scale), B, N, H, d)
    else:
        for z, h in slices:
            if not (0 <= z < B and 0 <= h < H):
                raise IndexError("slice out of range")
            lib.sigattn_oracle_fwd_slice(_p(q, _F), _p(k, _F), _p(v, _F), _p(o, _D), _p(seqlens, _I),
                                         _p(bias, _D), float(scale), B, N, H, d, int(z), int(h))
    return o


def bwd(q, k, v, d_o, seqlens, bias, scale: float,
        slices: Optional[Iterable[Tuple[int, int]]] = None):
    """(dQ, dK, dV) for every (z, h) slice, or only for the listed ones."""
    q, k, v, seqlens, bias, (B, N, H, d) = _common(q, k, v, seqlens, bias)
    d_o = _f32(d_o)
    if d_o.shape != q.shape:
        raise ValueError("d_o must have the shape of q")
    lib = _load()
    dq = np.zeros((B, N, H, d), dtype=np.float64)
    dk = np.zeros_like(dq)
    dv = np.zeros_like(dq)
    if slices is None:
        lib.sigattn_oracle_bwd(_p(q, _F), _p(k, _F), _p(v, _F), _p(d_o, _F), _p(dq, _D), _p(dk, _D), _p(dv, _D),
                               _p(seqlens, _I), _p(bias, _D), float(scale), B, N, H, d)
    else:
        for z, h in slices:
            if not (0 <= z < B and 0 <= h < H):
                raise IndexError("slice out of range")
            lib.sigattn_oracle_bwd_slice(_p(q, _F), _p(k, _F), _p(v, _F), _p(d_o, _F), _p(dq, _D), _p(dk, _D),
                                         _p(dv, _D), _p(seqlens, _I), _p(bias, _D), float(scale),
                                         B, N, H, d, int(z), int(h))
    return dq, dk, dv


def matrices(q, k, v, d_o, seqlens, bias, scale: float, z: int, h: int):
    """(P, dP, dS) of one slice as [N, N] arrays, zero outside the valid corner (tiny inputs only)."""
    q, k, v, seqlens, bias, (B, N, H, d) = _common(q, k, v, seqlens, bias)
    lib = _load()
    p = np.zeros((N, N), dtype=np.float64)
    dp = np.zeros_like(p)
    ds = np.zeros_like(p)
    if d_o is None:
        lib.sigattn_oracle_matrices(_p(q, _F), _p(k, _F), _p(v, _F), None, _p(p, _D), None, None,
                                    _p(seqlens, _I), _p(bias, _D), float(scale), B, N, H, d, int(z), int(h))
        return p, None, None
    d_o = _f32(d_o)
    lib.sigattn_oracle_matrices(_p(q, _F), _p(k, _F), _p(v, _F), _p(d_o, _F), _p(p, _D), _p(dp, _D), _p(ds, _D),
                                _p(seqlens, _I), _p(bias, _D), float(scale), B, N, H, d, int(z), int(h))
    return p, dp, ds


def _cross_common(q, k, v, seqlens_q, seqlens_k, bias):
    q, k, v = _f32(q), _f32(k), _f32(v)
    if k.shape != v.shape or q.shape[0] != k.shape[0] or q.shape[2:] != k.shape[2:]:
        raise ValueError("q is [B, L_q, H, d]; k and v are [B, L_k, H, d]")
    B, Lq, H, d = q.shape
    Lk = k.shape[1]
    seqlens_q = np.ascontiguousarray(seqlens_q, dtype=np.int32)
    seqlens_k = np.ascontiguousarray(seqlens_k, dtype=np.int32)
    bias = np.ascontiguousarray(bias, dtype=np.float64)
    if seqlens_q.shape != (B,) or seqlens_k.shape != (B,) or bias.shape != (B,):
        raise ValueError("seqlens_q, seqlens_k and bias must have shape [B]")
    return q, k, v, seqlens_q, seqlens_k, bias, (B, Lq, Lk, H, d)


def cross_fwd(q, k, v, seqlens_q, seqlens_k, bias, scale: float) -> np.ndarray:
    """O [B, L_q, H, d] with separate query and key lengths (appendix Alg. 1 as printed)."""
    q, k, v, sq, sk, bias, (B, Lq, Lk, H, d) = _cross_common(q, k, v, seqlens_q, seqlens_k, bias)
    o = np.zeros((B, Lq, H, d), dtype=np.float64)
    _load().sigattn_oracle_cross_fwd(_p(q, _F), _p(k, _F), _p(v, _F), _p(o, _D), _p(sq, _I), _p(sk, _I),
                                     _p(bias, _D), float(scale), B, Lq, Lk, H, d)
    return o


def cross_bwd(q, k, v, d_o, seqlens_q, seqlens_k, bias, scale: float):
    """(dQ [B,L_q,H,d], dK, dV [B,L_k,H,d], db [B]) with separate lengths (Alg. 2, Alg. 3; db: Sec. 3's
    learnable bias, db_z = sum over heads and valid pairs of dS)."""
    q, k, v, sq, sk, bias, (B, Lq, Lk, H, d) = _cross_common(q, k, v, seqlens_q, seqlens_k, bias)
    d_o = _f32(d_o)
    if d_o.shape != q.shape:
        raise ValueError("d_o must have the shape of q")
    dq = np.zeros((B, Lq, H, d), dtype=np.float64)
    dk = np.zeros((B, Lk, H, d), dtype=np.float64)
    dv = np.zeros_like(dk)
    db = np.zeros((B,), dtype=np.float64)
    _load().sigattn_oracle_cross_bwd(_p(q, _F), _p(k, _F), _p(v, _F), _p(d_o, _F), _p(dq, _D), _p(dk, _D),
                                     _p(dv, _D), _p(db, _D), _p(sq, _I), _p(sk, _I), _p(bias, _D), float(scale),
                                     B, Lq, Lk, H, d)
    return dq, dk, dv, db


# ----------------------------------------------------------------------------------------------
# Row-at-a-time evaluators (numpy fp64), for sampled checks on full-size workloads.
# ----------------------------------------------------------------------------------------------

def _sigma(x: np.ndarray) -> np.ndarray:
    """sigma(x) = 1 / (1 + exp(-x)), evaluated on the stable side of each sign."""
    out = np.empty_like(x)
    pos = x >= 0
    out[pos] = 1.0 / (1.0 + np.exp(-x[pos]))
    e = np.exp(x[~pos])
    out[~pos] = e / (1.0 + e)
    return out


def _n(seqlens, z, N) -> int:
    return int(min(max(int(seqlens[z]), 0), N))


def fwd_rows(q, k, v, seqlens, bias, scale: float, z: int, h: int, rows: Sequence[int]) -> np.ndarray:
    """O[z, i, h, :] for each i in rows -> [len(rows), d] float64 (zero for padded i)."""
    N, d = q.shape[1], q.shape[3]
    n = _n(seqlens, z, N)
    K = np.asarray(k[z, :n, h, :], dtype=np.float64)
    V = np.asarray(v[z, :n, h, :], dtype=np.float64)
    out = np.zeros((len(rows), d), dtype=np.float64)
    for r, i in enumerate(rows):
        if i >= n:
            continue
        x = float(scale) * (K @ np.asarray(q[z, i, h, :], dtype=np.float64)) + float(bias[z])
        out[r] = _sigma(x) @ V
    return out


def bwd_q_rows(q, k, v, d_o, seqlens, bias, scale: float, z: int, h: int, rows: Sequence[int]) -> np.ndarray:
    """dQ[z, i, h, :] for each i in rows -> [len(rows), d] float64."""
    N, d = q.shape[1], q.shape[3]
    n = _n(seqlens, z, N)
    K = np.asarray(k[z, :n, h, :], dtype=np.float64)
    V = np.asarray(v[z, :n, h, :], dtype=np.float64)
    out = np.zeros((len(rows), d), dtype=np.float64)
    for r, i in enumerate(rows):
        if i >= n:
            continue
        x = float(scale) * (K @ np.asarray(q[z, i, h, :], dtype=np.float64)) + float(bias[z])
        dp = V @ np.asarray(d_o[z, i, h, :], dtype=np.float64)
        ds = _sigma(x) * _sigma(-x) * dp
        out[r] = float(scale) * (ds @ K)
    return out


def bwd_kv_rows(q, k, v, d_o, seqlens, bias, scale: float, z: int, h: int, rows: Sequence[int]):
    """(dK[z, j, h, :], dV[z, j, h, :]) for each j in rows -> two [len(rows), d] float64 arrays."""
    N, d = q.shape[1], q.shape[3]
    n = _n(seqlens, z, N)
    Q = np.asarray(q[z, :n, h, :], dtype=np.float64)
    DO = np.asarray(d_o[z, :n, h, :], dtype=np.float64)
    dk = np.zeros((len(rows), d), dtype=np.float64)
    dv = np.zeros((len(rows), d), dtype=np.float64)
    for r, j in enumerate(rows):
        if j >= n:
            continue
        x = float(scale) * (Q @ np.asarray(k[z, j, h, :], dtype=np.float64)) + float(bias[z])
        p = _sigma(x)
        dp = DO @ np.asarray(v[z, j, h, :], dtype=np.float64)
        ds = p * _sigma(-x) * dp
        dv[r] = p @ DO
        dk[r] = float(scale) * (ds @ Q)
    return dk, dv


def valid_flops(seqlens, H: int, d: int, N: Optional[int] = None):
    """(forward, backward) FLOPs over valid tokens only.

    Paper appendix "FLOP Calculation": forward = 4 b h n^2 d (two matmuls of
    2 n^2 d each), backward = 2.5 x forward; with padding n counts valid tokens,
    so a jagged batch uses sum_z n_z^2 in place of b n^2.
    """
    n = np.asarray(seqlens, dtype=np.int64)
    if N is not None:
        n = np.clip(n, 0, N)
    pairs = int(np.sum(n * n))
    f = 4 * H * d * pairs
    return f, (5 * f) // 2
