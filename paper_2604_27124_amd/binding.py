"""ctypes binding over libsigattn.so -- argument marshalling only.

The functions carry the names of the C ABI (include/sigmoid_attn.h).  Tensors are torch
CUDA(=HIP) bf16 tensors used purely as device memory; every step of the computation runs in
the library's kernels.  There is no CPU path: a missing library is an error.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libsigattn.so")

SIGATTN_OK = 0
SIGATTN_ERR_INVALID_ARG = -1
SIGATTN_ERR_UNSUPPORTED_D = -2
SIGATTN_ERR_MISALIGNED = -3
SIGATTN_ERR_WORKSPACE = -4
SIGATTN_ERR_LAUNCH = -5
SIGATTN_ERR_TOO_LARGE = -6

EXPORTS = ("sigmoid_attn_version", "sigmoid_attn_strerror", "sigmoid_attn_fwd", "sigmoid_attn_bwd",
           "sigmoid_attn_bwd_dq", "sigmoid_attn_bwd_dkdv", "sigmoid_attn_bwd_workspace_bytes",
           "sigmoid_attn_cross_fwd", "sigmoid_attn_cross_bwd",
           "sigmoid_attn_bwd_dq_dbias", "sigmoid_attn_bwd_dq_dbias_workspace_bytes",
           "sigmoid_attn_cross_bwd_dq_dbias", "sigmoid_attn_cross_bwd_dq_dbias_workspace_bytes",
           "sigmoid_attn_bwd_dq_dbias_static")

_lib = None


class SigAttnError(RuntimeError):
    def __init__(self, code: int):
        self.code = code
        super().__init__(f"libsigattn error {code}: {sigmoid_attn_strerror(code)}")


def load() -> ctypes.CDLL:
    """The loaded C library (raises if it has not been built)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_27124_amd.build` "
                               "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, ci, cf, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_float, ctypes.c_size_t
        lib.sigmoid_attn_version.argtypes = []
        lib.sigmoid_attn_version.restype = ci
        lib.sigmoid_attn_strerror.argtypes = [ci]
        lib.sigmoid_attn_strerror.restype = ctypes.c_char_p
        lib.sigmoid_attn_fwd.argtypes = [vp, vp, vp, vp, vp, vp, cf, ci, ci, ci, ci, vp]
        lib.sigmoid_attn_fwd.restype = ci
        lib.sigmoid_attn_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, cf, ci, ci, ci, ci, vp, sz, vp]
        lib.sigmoid_attn_bwd.restype = ci
        lib.sigmoid_attn_bwd_dq.argtypes = [vp, vp, vp, vp, vp, vp, vp, cf, ci, ci, ci, ci, vp]
        lib.sigmoid_attn_bwd_dq.restype = ci
        lib.sigmoid_attn_bwd_dkdv.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, cf, ci, ci, ci, ci, vp]
        lib.sigmoid_attn_bwd_dkdv.restype = ci
        lib.sigmoid_attn_cross_fwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, cf, ci, ci, ci, ci, ci, vp]
        lib.sigmoid_attn_cross_fwd.restype = ci
        lib.sigmoid_attn_cross_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, cf, ci, ci, ci, ci, ci, vp]
        lib.sigmoid_attn_cross_bwd.restype = ci
        lib.sigmoid_attn_bwd_dq_dbias.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, cf, ci, ci, ci, ci, vp, sz, vp]
        lib.sigmoid_attn_bwd_dq_dbias.restype = ci
        lib.sigmoid_attn_bwd_dq_dbias_workspace_bytes.argtypes = [ci, ci, ci, ci]
        lib.sigmoid_attn_bwd_dq_dbias_workspace_bytes.restype = sz
        lib.sigmoid_attn_cross_bwd_dq_dbias.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, vp, cf, ci, ci, ci, ci, ci, vp, sz, vp]
        lib.sigmoid_attn_cross_bwd_dq_dbias.restype = ci
        lib.sigmoid_attn_cross_bwd_dq_dbias_workspace_bytes.argtypes = [ci, ci, ci, ci, ci]
        lib.sigmoid_attn_cross_bwd_dq_dbias_workspace_bytes.restype = sz
        lib.sigmoid_attn_bwd_dq_dbias_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, cf, ci, ci, ci, ci, vp]
        lib.sigmoid_attn_bwd_dq_dbias_static.restype = ci
        lib.sigmoid_attn_bwd_workspace_bytes.argtypes = [ci, ci, ci, ci]
        lib.sigmoid_attn_bwd_workspace_bytes.restype = sz
        _lib = lib
    return _lib


def sigmoid_attn_version() -> int:
    return int(load().sigmoid_attn_version())


def sigmoid_attn_strerror(code: int) -> str:
    return load().sigmoid_attn_strerror(int(code)).decode()


def sigmoid_attn_bwd_workspace_bytes(B: int, N_max: int, H: int, d: int) -> int:
    return int(load().sigmoid_attn_bwd_workspace_bytes(B, N_max, H, d))


def _check(t, name: str, shape=None):
    import torch
    if not (t.is_cuda and t.dtype == torch.bfloat16 and t.is_contiguous() and t.dim() == 4):
        raise ValueError(f"{name} must be a contiguous CUDA bf16 tensor of shape [B, N_max, H, d]")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {tuple(shape)}")


def _check_vec(t, name: str, B: int, dtype):
    if not (t.is_cuda and t.dtype == dtype and t.is_contiguous() and tuple(t.shape) == (B,)):
        raise ValueError(f"{name} must be a contiguous CUDA {dtype} tensor of shape [B]")


def _stream_ptr(stream) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def sigmoid_attn_fwd(q, k, v, seqlens, bias, scale: float, out=None, stream=None):
    """O = sigmoid(scale * Q K^T + bias) V over valid tokens; returns `out` (allocated if None)."""
    import torch
    _check(q, "q")
    _check(k, "k", q.shape)
    _check(v, "v", q.shape)
    B, N, H, d = q.shape
    _check_vec(seqlens, "seqlens", B, torch.int32)
    _check_vec(bias, "bias", B, torch.float32)
    if out is None:
        out = torch.empty_like(q)
    _check(out, "out", q.shape)
    rc = load().sigmoid_attn_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(), seqlens.data_ptr(),
                                 bias.data_ptr(), float(scale), B, N, H, d, _stream_ptr(stream))
    if rc != SIGATTN_OK:
        raise SigAttnError(rc)
    return out


def sigmoid_attn_bwd(q, k, v, d_o, seqlens, bias, scale: float, dq=None, dk=None, dv=None, workspace=None,
                     stream=None) -> Tuple:
    """(dQ, dK, dV) from the forward inputs and dO; outputs and workspace are allocated if None."""
    import torch
    _check(q, "q")
    for t, name in ((k, "k"), (v, "v"), (d_o, "d_o")):
        _check(t, name, q.shape)
    B, N, H, d = q.shape
    _check_vec(seqlens, "seqlens", B, torch.int32)
    _check_vec(bias, "bias", B, torch.float32)
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(q) if dk is None else dk
    dv = torch.empty_like(q) if dv is None else dv
    for t, name in ((dq, "dq"), (dk, "dk"), (dv, "dv")):
        _check(t, name, q.shape)
    need = sigmoid_attn_bwd_workspace_bytes(B, N, H, d)
    if workspace is None and need > 0:
        workspace = torch.empty(need, dtype=torch.uint8, device=q.device)
    ws_ptr = 0 if workspace is None else workspace.data_ptr()
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    rc = load().sigmoid_attn_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), d_o.data_ptr(), dq.data_ptr(),
                                 dk.data_ptr(), dv.data_ptr(), seqlens.data_ptr(), bias.data_ptr(), float(scale),
                                 B, N, H, d, ws_ptr, ws_bytes, _stream_ptr(stream))
    if rc != SIGATTN_OK:
        raise SigAttnError(rc)
    return dq, dk, dv


def sigmoid_attn_bwd_dq(q, k, v, d_o, seqlens, bias, scale: float, dq=None, stream=None):
    """dQ alone (the query-gradient kernel)."""
    import torch
    _check(q, "q")
    for t, name in ((k, "k"), (v, "v"), (d_o, "d_o")):
        _check(t, name, q.shape)
    B, N, H, d = q.shape
    _check_vec(seqlens, "seqlens", B, torch.int32)
    _check_vec(bias, "bias", B, torch.float32)
    dq = torch.empty_like(q) if dq is None else dq
    _check(dq, "dq", q.shape)
    rc = load().sigmoid_attn_bwd_dq(q.data_ptr(), k.data_ptr(), v.data_ptr(), d_o.data_ptr(), dq.data_ptr(),
                                    seqlens.data_ptr(), bias.data_ptr(), float(scale), B, N, H, d,
                                    _stream_ptr(stream))
    if rc != SIGATTN_OK:
        raise SigAttnError(rc)
    return dq


def sigmoid_attn_bwd_dkdv(q, k, v, d_o, seqlens, bias, scale: float, dk=None, dv=None, stream=None):
    """dK and dV alone (the key/value-gradient kernel)."""
    import torch
    _check(q, "q")
    for t, name in ((k, "k"), (v, "v"), (d_o, "d_o")):
        _check(t, name, q.shape)
    B, N, H, d = q.shape
    _check_vec(seqlens, "seqlens", B, torch.int32)
    _check_vec(bias, "bias", B, torch.float32)
    dk = torch.empty_like(q) if dk is None else dk
    dv = torch.empty_like(q) if dv is None else dv
    _check(dk, "dk", q.shape)
    _check(dv, "dv", q.shape)
    rc = load().sigmoid_attn_bwd_dkdv(q.data_ptr(), k.data_ptr(), v.data_ptr(), d_o.data_ptr(), dk.data_ptr(),
                                      dv.data_ptr(), seqlens.data_ptr(), bias.data_ptr(), float(scale), B, N, H, d,
                                      _stream_ptr(stream))
    if rc != SIGATTN_OK:
        raise SigAttnError(rc)
    return dk, dv


def _check_cross(q, k, v):
    _check(q, "q")
    _check(k, "k")
    _check(v, "v", k.shape)
    if q.shape[0] != k.shape[0] or q.shape[2:] != k.shape[2:]:
        raise ValueError("q is [B, L_q, H, d]; k and v are [B, L_k, H, d]")


def sigmoid_attn_cross_fwd(q, k, v, seqlens_q, seqlens_k, bias, scale: float, out=None, stream=None):
    """Forward pass with separate query and key lengths: q [B, L_q, H, d]; k, v [B, L_k, H, d]."""
    import torch
    _check_cross(q, k, v)
    B, Lq, H, d = q.shape
    Lk = k.shape[1]
    _check_vec(seqlens_q, "seqlens_q", B, torch.int32)
    _check_vec(seqlens_k, "seqlens_k", B, torch.int32)
    _check_vec(bias, "bias", B, torch.float32)
    if out is None:
        out = torch.empty_like(q)
    _check(out, "out", q.shape)
    rc = load().sigmoid_attn_cross_fwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), out.data_ptr(),
                                       seqlens_q.data_ptr(), seqlens_k.data_ptr(), bias.data_ptr(), float(scale),
                                       B, Lq, Lk, H, d, _stream_ptr(stream))
    if rc != SIGATTN_OK:
        raise SigAttnError(rc)
    return out


def sigmoid_attn_cross_bwd(q, k, v, d_o, seqlens_q, seqlens_k, bias, scale: float, dq=None, dk=None, dv=None,
                           stream=None) -> Tuple:
    """(dQ [B, L_q, H, d], dK, dV [B, L_k, H, d]) with separate query and key lengths."""
    import torch
    _check_cross(q, k, v)
    _check(d_o, "d_o", q.shape)
    B, Lq, H, d = q.shape
    Lk = k.shape[1]
    _check_vec(seqlens_q, "seqlens_q", B, torch.int32)
    _check_vec(seqlens_k, "seqlens_k", B, torch.int32)
    _check_vec(bias, "bias", B, torch.float32)
    dq = torch.empty_like(q) if dq is None else dq
    dk = torch.empty_like(k) if dk is None else dk
    dv = torch.empty_like(k) if dv is None else dv
    _check(dq, "dq", q.shape)
    _check(dk, "dk", k.shape)
    _check(dv, "dv", k.shape)
    rc = load().sigmoid_attn_cross_bwd(q.data_ptr(), k.data_ptr(), v.data_ptr(), d_o.data_ptr(), dq.data_ptr(),
                                       dk.data_ptr(), dv.data_ptr(), seqlens_q.data_ptr(), seqlens_k.data_ptr(),
                                       bias.data_ptr(), float(scale), B, Lq, Lk, H, d, _stream_ptr(stream))
    if rc != SIGATTN_OK:
        raise SigAttnError(rc)
    return dq, dk, dv


def sigmoid_attn_bwd_dq_dbias_workspace_bytes(B: int, N_max: int, H: int, d: int) -> int:
    return int(load().sigmoid_attn_bwd_dq_dbias_workspace_bytes(B, N_max, H, d))


def sigmoid_attn_bwd_dq_dbias(q, k, v, d_o, seqlens, bias, scale: float, dq=None, dbias=None, workspace=None,
                              stream=None):
    """(dQ, dbias [B] float32): the query gradient together with the gradient of the per-sequence bias."""
    import torch
    _check(q, "q")
    for t, name in ((k, "k"), (v, "v"), (d_o, "d_o")):
        _check(t, name, q.shape)
    B, N, H, d = q.shape
    _check_vec(seqlens, "seqlens", B, torch.int32)
    _check_vec(bias, "bias", B, torch.float32)
    dq = torch.empty_like(q) if dq is None else dq
    _check(dq, "dq", q.shape)
    dbias = torch.empty(B, dtype=torch.float32, device=q.device) if dbias is None else dbias
    _check_vec(dbias, "dbias", B, torch.float32)
    need = sigmoid_attn_bwd_dq_dbias_workspace_bytes(B, N, H, d)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    rc = load().sigmoid_attn_bwd_dq_dbias(q.data_ptr(), k.data_ptr(), v.data_ptr(), d_o.data_ptr(), dq.data_ptr(),
                                          dbias.data_ptr(), seqlens.data_ptr(), bias.data_ptr(), float(scale),
                                          B, N, H, d, workspace.data_ptr(),
                                          workspace.numel() * workspace.element_size(), _stream_ptr(stream))
    if rc != SIGATTN_OK:
        raise SigAttnError(rc)
    return dq, dbias


def sigmoid_attn_bwd_dq_dbias_static(q, k, v, d_o, seqlens, bias, scale: float, dq, dbias, stream=None):
    """sigmoid_attn_bwd_dq_dbias without a workspace and without any allocation: the caller passes both
    outputs (dq like q, dbias float32 [B]); the partial sums go to the library's own static device array."""
    import torch
    _check(q, "q")
    for t, name in ((k, "k"), (v, "v"), (d_o, "d_o"), (dq, "dq")):
        _check(t, name, q.shape)
    B, N, H, d = q.shape
    _check_vec(seqlens, "seqlens", B, torch.int32)
    _check_vec(bias, "bias", B, torch.float32)
    _check_vec(dbias, "dbias", B, torch.float32)
    rc = load().sigmoid_attn_bwd_dq_dbias_static(q.data_ptr(), k.data_ptr(), v.data_ptr(), d_o.data_ptr(),
                                                 dq.data_ptr(), dbias.data_ptr(), seqlens.data_ptr(),
                                                 bias.data_ptr(), float(scale), B, N, H, d, _stream_ptr(stream))
    if rc != SIGATTN_OK:
        raise SigAttnError(rc)
    return dq, dbias


def sigmoid_attn_cross_bwd_dq_dbias_workspace_bytes(B: int, L_q: int, L_k: int, H: int, d: int) -> int:
    return int(load().sigmoid_attn_cross_bwd_dq_dbias_workspace_bytes(B, L_q, L_k, H, d))


def sigmoid_attn_cross_bwd_dq_dbias(q, k, v, d_o, seqlens_q, seqlens_k, bias, scale: float, dq=None, dbias=None,
                                    workspace=None, stream=None):
    """(dQ, dbias [B] float32) with separate query and key lengths."""
    import torch
    _check_cross(q, k, v)
    B, L_q, H, d = q.shape
    L_k = k.shape[1]
    _check(d_o, "d_o", q.shape)
    _check_vec(seqlens_q, "seqlens_q", B, torch.int32)
    _check_vec(seqlens_k, "seqlens_k", B, torch.int32)
    _check_vec(bias, "bias", B, torch.float32)
    dq = torch.empty_like(q) if dq is None else dq
    _check(dq, "dq", q.shape)
    dbias = torch.empty(B, dtype=torch.float32, device=q.device) if dbias is None else dbias
    _check_vec(dbias, "dbias", B, torch.float32)
    need = sigmoid_attn_cross_bwd_dq_dbias_workspace_bytes(B, L_q, L_k, H, d)
    if workspace is None:
        workspace = torch.empty(max(need, 16), dtype=torch.uint8, device=q.device)
    rc = load().sigmoid_attn_cross_bwd_dq_dbias(q.data_ptr(), k.data_ptr(), v.data_ptr(), d_o.data_ptr(),
                                                dq.data_ptr(), dbias.data_ptr(), seqlens_q.data_ptr(),
                                                seqlens_k.data_ptr(), bias.data_ptr(), float(scale), B, L_q, L_k, H, d,
                                                workspace.data_ptr(), workspace.numel() * workspace.element_size(),
                                                _stream_ptr(stream))
    if rc != SIGATTN_OK:
        raise SigAttnError(rc)
    return dq, dbias
