"""Pins for the oracle's cross-attention functions (separate query / key lengths, appendix Alg. 1-3 as
printed with n_q, n_k, L_q, L_k) and for the bias gradient (Sec. 3: the bias may be learnable).
CPU only: brute force, torch fp64 autograd, finite differences, closed forms, reduction to the
self-attention oracle, empty sides."""
import math

import numpy as np
import pytest
import torch

import oracle
from paper_2604_27124_amd import workloads as W


def draw(B, Lq, Lk, H, d, seed, std=1.0):
    rng = np.random.default_rng(seed)
    mk = lambda L: W.round_to_bf16((rng.standard_normal((B, L, H, d)) * std).astype(np.float32))
    return mk(Lq), mk(Lk), mk(Lk), mk(Lq)


def brute(q, k, v, g, nq, nk, bias, scale):
    B, Lq, H, d = q.shape
    Lk = k.shape[1]
    q, k, v, g = (np.asarray(a, np.float64) for a in (q, k, v, g))
    o = np.zeros((B, Lq, H, d)); dq = np.zeros_like(o)
    dk = np.zeros((B, Lk, H, d)); dv = np.zeros_like(dk); db = np.zeros(B)
    for z in range(B):
        for h in range(H):
            for i in range(nq[z]):
                for j in range(nk[z]):
                    x = scale * sum(q[z, i, h, c] * k[z, j, h, c] for c in range(d)) + bias[z]
                    p = 1.0 / (1.0 + math.exp(-x))
                    dp = sum(g[z, i, h, c] * v[z, j, h, c] for c in range(d))
                    ds = p * (1.0 - p) * dp
                    db[z] += ds
                    for c in range(d):
                        o[z, i, h, c] += p * v[z, j, h, c]
                        dv[z, j, h, c] += p * g[z, i, h, c]
                        dq[z, i, h, c] += scale * ds * k[z, j, h, c]
                        dk[z, j, h, c] += scale * ds * q[z, i, h, c]
    return o, dq, dk, dv, db


@pytest.mark.parametrize("nq,nk", [((5, 3), (4, 6)), ((1, 5), (6, 1)), ((0, 2), (3, 0))])
def test_brute_force_tiny(nq, nk):
    q, k, v, g = draw(2, 5, 6, 2, 3, seed=11)
    bias, scale = [-0.7, 0.3], 0.6
    o = oracle.cross_fwd(q, k, v, nq, nk, bias, scale)
    dq, dk, dv, db = oracle.cross_bwd(q, k, v, g, nq, nk, bias, scale)
    for got, ref in zip((o, dq, dk, dv, db), brute(q, k, v, g, nq, nk, bias, scale)):
        assert np.allclose(got, ref, rtol=1e-12, atol=1e-14)


def test_equal_lengths_reduce_to_self_attention_oracle():
    w = W.make(3, 19, 2, 8, (19, 11, 0), seed=5, qkv_std=1.3)
    o = oracle.cross_fwd(w.q, w.k, w.v, w.seqlens, w.seqlens, w.bias, w.scale)
    dq, dk, dv, _ = oracle.cross_bwd(w.q, w.k, w.v, w.d_o, w.seqlens, w.seqlens, w.bias, w.scale)
    assert np.array_equal(o, oracle.fwd(w.q, w.k, w.v, w.seqlens, w.bias, w.scale))
    for a, b in zip((dq, dk, dv), oracle.bwd(w.q, w.k, w.v, w.d_o, w.seqlens, w.bias, w.scale)):
        assert np.array_equal(a, b)


def test_against_torch_autograd_fp64_including_bias():
    B, Lq, Lk, H, d = 2, 21, 34, 2, 8
    q, k, v, g = draw(B, Lq, Lk, H, d, seed=3, std=1.4)
    nq, nk = (21, 9), (30, 34)
    bias, scale = np.array([-1.2, -2.0]), 0.31
    o = oracle.cross_fwd(q, k, v, nq, nk, bias, scale)
    dq, dk, dv, db = oracle.cross_bwd(q, k, v, g, nq, nk, bias, scale)
    for z in range(B):
        tq = torch.tensor(q[z, :nq[z]], dtype=torch.float64, requires_grad=True)
        tk = torch.tensor(k[z, :nk[z]], dtype=torch.float64, requires_grad=True)
        tv = torch.tensor(v[z, :nk[z]], dtype=torch.float64, requires_grad=True)
        tb = torch.tensor(bias[z], dtype=torch.float64, requires_grad=True)
        s = torch.einsum("ihc,jhc->hij", tq, tk) * scale + tb
        to = torch.einsum("hij,jhc->ihc", torch.sigmoid(s), tv)
        to.backward(torch.tensor(g[z, :nq[z]], dtype=torch.float64))
        assert np.allclose(o[z, :nq[z]], to.detach().numpy(), rtol=1e-11, atol=1e-13)
        assert np.allclose(dq[z, :nq[z]], tq.grad.numpy(), rtol=1e-11, atol=1e-13)
        assert np.allclose(dk[z, :nk[z]], tk.grad.numpy(), rtol=1e-11, atol=1e-13)
        assert np.allclose(dv[z, :nk[z]], tv.grad.numpy(), rtol=1e-11, atol=1e-13)
        assert np.isclose(db[z], float(tb.grad), rtol=1e-11, atol=1e-13)
        assert np.all(o[z, nq[z]:] == 0) and np.all(dq[z, nq[z]:] == 0)
        assert np.all(dk[z, nk[z]:] == 0) and np.all(dv[z, nk[z]:] == 0)


def test_bias_gradient_by_finite_differences():
    q, k, v, g = draw(2, 6, 9, 2, 4, seed=8)
    nq, nk, scale = (6, 4), (7, 9), 0.5
    bias = np.array([-0.5, -1.5])
    _, _, _, db = oracle.cross_bwd(q, k, v, g, nq, nk, bias, scale)
    for z in range(2):
        def loss(b):
            bb = bias.copy(); bb[z] = b
            return float(np.sum(oracle.cross_fwd(q, k, v, nq, nk, bb, scale) * g.astype(np.float64)))
        h = 1e-3
        c = lambda hh: (loss(bias[z] + hh) - loss(bias[z] - hh)) / (2 * hh)
        fd = (4 * c(h / 2) - c(h)) / 3
        assert abs(fd - db[z]) <= 1e-9 + 1e-8 * abs(db[z])


def test_zero_query_closed_form_with_two_lengths():
    # Q = 0: every valid weight is s = sigma(b).  O_i = s sum_{j<n_k} v_j;  dV_j = s sum_{i<n_q} dO_i;
    # db = s (1 - s) sum_h sum_{i<n_q, j<n_k} <dO_i, v_j>;  dK = 0.
    B, Lq, Lk, H, d = 1, 7, 5, 2, 4
    q, k, v, g = draw(B, Lq, Lk, H, d, seed=2)
    q[:] = 0
    nq, nk, b, scale = (6,), (4,), -math.log(4.0), 0.5
    s = 1.0 / 5.0
    o = oracle.cross_fwd(q, k, v, nq, nk, [b], scale)
    dq, dk, dv, db = oracle.cross_bwd(q, k, v, g, nq, nk, [b], scale)
    vs = v[0, :4].astype(np.float64).sum(axis=0)            # [H, d]
    gs = g[0, :6].astype(np.float64).sum(axis=0)
    assert np.allclose(o[0, :6], s * vs[None], rtol=1e-13)
    assert np.allclose(dv[0, :4], s * gs[None], rtol=1e-13)
    assert np.all(dk == 0.0)
    assert np.isclose(db[0], s * (1 - s) * float(np.sum(gs * vs)), rtol=1e-12)


def test_empty_sides():
    q, k, v, g = draw(2, 4, 6, 1, 4, seed=4)
    o = oracle.cross_fwd(q, k, v, (4, 0), (0, 6), [0.1, 0.2], 0.5)
    dq, dk, dv, db = oracle.cross_bwd(q, k, v, g, (4, 0), (0, 6), [0.1, 0.2], 0.5)
    for a in (o, dq, dk, dv, db):
        assert np.all(a == 0.0)
