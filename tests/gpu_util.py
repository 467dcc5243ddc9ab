"""Helpers for the GPU parity tests: device upload, the error norm, oracle comparison."""
from __future__ import annotations

import numpy as np
import torch

import oracle
from paper_2604_27124_amd import binding
from paper_2604_27124_amd import workloads as W

FWD_TOL = 1e-2     # max |gpu - ref| / max |ref| per (z, h) slice, forward
BWD_TOL = 2e-2     # same norm, each of dQ, dK, dV


def to_dev(a: np.ndarray) -> torch.Tensor:
    """bf16-valued float32 numpy -> bf16 device tensor, bit-exact."""
    bits = W.bf16_bits(a).view(np.int16)
    return torch.from_numpy(bits).cuda().view(torch.bfloat16)


def to_host(t: torch.Tensor) -> np.ndarray:
    """bf16 device tensor -> float32 numpy, bit-exact."""
    return W.bits_to_f32(t.view(torch.int16).cpu().numpy())


class Dev:
    def __init__(self, w: W.Workload):
        self.w = w
        self.q, self.k, self.v, self.d_o = (to_dev(x) for x in (w.q, w.k, w.v, w.d_o))
        self.seqlens = torch.from_numpy(np.ascontiguousarray(w.seqlens, dtype=np.int32)).cuda()
        self.bias = torch.from_numpy(np.ascontiguousarray(w.bias, dtype=np.float32)).cuda()

    def fwd(self, poison=True):
        out = torch.full_like(self.q, float("nan")) if poison else None
        o = binding.sigmoid_attn_fwd(self.q, self.k, self.v, self.seqlens, self.bias, self.w.scale, out=out)
        torch.cuda.synchronize()
        return o

    def bwd(self, poison=True):
        outs = [torch.full_like(self.q, float("nan")) for _ in range(3)] if poison else [None] * 3
        r = binding.sigmoid_attn_bwd(self.q, self.k, self.v, self.d_o, self.seqlens, self.bias, self.w.scale,
                                     dq=outs[0], dk=outs[1], dv=outs[2])
        torch.cuda.synchronize()
        return r


def slice_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref| over one slice's valid rows (0 if both are all zero)."""
    den = float(np.max(np.abs(ref))) if ref.size else 0.0
    num = float(np.max(np.abs(got.astype(np.float64) - ref))) if ref.size else 0.0
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den


def check_slices(name, got: np.ndarray, ref: np.ndarray, seqlens, slices, tol) -> float:
    """Compare [B, N, H, d] arrays on the listed (z, h) slices; padded rows must be exact zeros."""
    worst = 0.0
    assert np.all(np.isfinite(got)), f"{name}: non-finite values in the output"
    for z, h in slices:
        n = int(seqlens[z])
        assert np.all(got[z, n:, h] == 0.0), f"{name}: padded rows of slice {(z, h)} are not zero"
        e = slice_err(got[z, :n, h], ref[z, :n, h])
        worst = max(worst, e)
        assert e <= tol, f"{name}: slice {(z, h)} n={n} error {e:.3e} > {tol}"
    return worst


def all_slices(w):
    return [(z, h) for z in range(w.B) for h in range(w.H)]


def check_against_oracle(w: W.Workload, slices=None, fwd=True, bwd=True, dev: Dev | None = None):
    """Run the HIP path on w and compare whole (z, h) slices with the C oracle."""
    dev = dev or Dev(w)
    slices = all_slices(w) if slices is None else slices
    res = {}
    if fwd:
        o = to_host(dev.fwd())
        ref = oracle.fwd(w.q, w.k, w.v, w.seqlens, w.bias, w.scale, slices=slices)
        res["o"] = check_slices("O", o, ref, w.seqlens, slices, FWD_TOL)
        _check_untouched_padding(o, w, "O")
    if bwd:
        dq, dk, dv = (to_host(t) for t in dev.bwd())
        rq, rk, rv = oracle.bwd(w.q, w.k, w.v, w.d_o, w.seqlens, w.bias, w.scale, slices=slices)
        res["dq"] = check_slices("dQ", dq, rq, w.seqlens, slices, BWD_TOL)
        res["dk"] = check_slices("dK", dk, rk, w.seqlens, slices, BWD_TOL)
        res["dv"] = check_slices("dV", dv, rv, w.seqlens, slices, BWD_TOL)
        for a, nm in ((dq, "dQ"), (dk, "dK"), (dv, "dV")):
            _check_untouched_padding(a, w, nm)
    return res


def _check_untouched_padding(a: np.ndarray, w: W.Workload, name: str):
    """Every padded row of every slice is an exact zero (the outputs were NaN-poisoned before the call)."""
    for z in range(w.B):
        n = int(w.seqlens[z])
        assert np.all(a[z, n:] == 0.0), f"{name}: padded rows of sequence {z} not written as zero"
