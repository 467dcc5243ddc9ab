"""GPU parity of the cross-attention entry points (separate query / key lengths; appendix Alg. 1-3 as
printed) against the fp64 oracle: element by element on whole tensors, over shapes that straddle the
kernels' tile sizes on either side, with empty sides and with L_q != L_k."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_27124_amd import binding
from paper_2604_27124_amd import workloads as W
from gpu_util import BWD_TOL, FWD_TOL, to_dev, to_host

pytestmark = pytest.mark.gpu


def draw(B, Lq, Lk, H, d, seed, std=1.0):
    rng = np.random.default_rng(seed)
    mk = lambda L, s: W.round_to_bf16((rng.standard_normal((B, L, H, d)) * s).astype(np.float32))
    return mk(Lq, std), mk(Lk, std), mk(Lk, std), mk(Lq, 1.0)


def err(got, ref):
    den = float(np.abs(ref).max())
    return float(np.abs(got - ref).max()) / den if den > 0 else float(np.abs(got).max())


def run_case(B, Lq, Lk, H, d, nq, nk, seed=0, std=1.0):
    q, k, v, g = draw(B, Lq, Lk, H, d, seed, std)
    nq, nk = np.asarray(nq, np.int32), np.asarray(nk, np.int32)
    bias = (-np.log(np.maximum(nk, 1))).astype(np.float32)
    scale = 1.0 / np.sqrt(d)
    dq_, dk_, dv_, g_ = to_dev(q), to_dev(k), to_dev(v), to_dev(g)
    sq, sk, b = torch.from_numpy(nq).cuda(), torch.from_numpy(nk).cuda(), torch.from_numpy(bias).cuda()
    poison = lambda t: torch.full_like(t, float("nan"))
    o = binding.sigmoid_attn_cross_fwd(dq_, dk_, dv_, sq, sk, b, scale, out=poison(dq_))
    gq, gk, gv = binding.sigmoid_attn_cross_bwd(dq_, dk_, dv_, g_, sq, sk, b, scale, dq=poison(dq_), dk=poison(dk_),
                                                dv=poison(dk_))
    torch.cuda.synchronize()
    ro = oracle.cross_fwd(q, k, v, nq, nk, bias, scale)
    rq, rk, rv, _ = oracle.cross_bwd(q, k, v, g, nq, nk, bias, scale)
    worst = {}
    for name, got, ref, lens, tol in (("o", o, ro, nq, FWD_TOL), ("dq", gq, rq, nq, BWD_TOL),
                                      ("dk", gk, rk, nk, BWD_TOL), ("dv", gv, rv, nk, BWD_TOL)):
        got = to_host(got)
        assert np.all(np.isfinite(got)), name
        w = 0.0
        for z in range(B):
            n = int(lens[z])
            assert np.all(got[z, n:] == 0.0), f"{name}: padded rows of sequence {z} not zero"
            for h in range(H):
                if n == 0 or np.abs(ref[z, :n, h]).max() == 0:
                    assert np.all(got[z, :n, h] == 0.0)
                    continue
                e = err(got[z, :n, h], ref[z, :n, h])
                assert e <= tol, f"{name} slice {(z, h)} (n_q={nq[z]}, n_k={nk[z]}): error {e:.3e} > {tol}"
                w = max(w, e)
        worst[name] = w
    print("cross", (B, Lq, Lk, H, d), nq.tolist(), nk.tolist(), worst, flush=True)


@pytest.mark.parametrize("nq,nk", [((300, 17), (129, 600)), ((1, 256), (512, 1)), ((0, 64), (100, 0)),
                                   ((257, 255), (63, 65)), ((300, 300), (640, 640))])
def test_cross_d64(nq, nk):
    run_case(2, 300, 640, 2, 64, nq, nk, seed=1)


@pytest.mark.parametrize("nq,nk", [((130, 40), (70, 200)), ((200, 0), (1, 77))])
def test_cross_d128(nq, nk):
    run_case(2, 200, 200, 2, 128, nq, nk, seed=2)


def test_cross_long_keys_short_queries_d64():
    run_case(1, 128, 5000, 2, 64, (100,), (4999,), seed=3, std=1.2)


def test_cross_equals_self_when_lengths_agree():
    w = W.make(2, 300, 2, 64, (300, 173), seed=4)
    q, k, v, g = to_dev(w.q), to_dev(w.k), to_dev(w.v), to_dev(w.d_o)
    s, b = torch.from_numpy(w.seqlens).cuda(), torch.from_numpy(w.bias).cuda()
    o1 = binding.sigmoid_attn_fwd(q, k, v, s, b, w.scale)
    o2 = binding.sigmoid_attn_cross_fwd(q, k, v, s, s, b, w.scale)
    a = binding.sigmoid_attn_bwd(q, k, v, g, s, b, w.scale)
    c = binding.sigmoid_attn_cross_bwd(q, k, v, g, s, s, b, w.scale)
    torch.cuda.synchronize()
    assert torch.equal(o1.view(torch.int16), o2.view(torch.int16))
    for x, y in zip(a, c):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))


@pytest.mark.parametrize("d", [64, 128])
def test_cross_many_sequences(d):
    # more than 256 sequences (tile-count ranking of the work mapping) with different lengths on the two
    # sides: the owner side is ranked, the streamed length is looked up per sequence
    B = 300
    rng = np.random.default_rng(7)
    nq = rng.integers(0, 291, size=B); nk = rng.integers(0, 151, size=B)
    nq[:3] = (290, 0, 1); nk[:3] = (150, 150, 0)
    run_case(B, 290, 150, 1, d, nq, nk, seed=5)


def test_dq_dbias_many_sequences():
    # the bias-gradient entry point over more than 256 sequences: one partial per workgroup, summed per sequence
    B = 300
    rng = np.random.default_rng(8)
    lens = rng.integers(0, 301, size=B)
    w = W.make(B, 300, 2, 64, lens, seed=6)
    w.v[:] = np.abs(w.v); w.d_o[:] = np.abs(w.d_o)          # every dS >= 0: the sum does not cancel
    q, k, v, g = to_dev(w.q), to_dev(w.k), to_dev(w.v), to_dev(w.d_o)
    s, b = torch.from_numpy(w.seqlens).cuda(), torch.from_numpy(w.bias).cuda()
    dq, db = binding.sigmoid_attn_bwd_dq_dbias(q, k, v, g, s, b, w.scale)
    dq_only = binding.sigmoid_attn_bwd_dq(q, k, v, g, s, b, w.scale)
    torch.cuda.synchronize()
    assert torch.equal(dq.view(torch.int16), dq_only.view(torch.int16))
    _, _, _, ref = oracle.cross_bwd(w.q, w.k, w.v, w.d_o, w.seqlens, w.seqlens, w.bias, w.scale)
    got = db.cpu().numpy().astype(np.float64)
    assert np.all(got[lens == 0] == 0.0)
    assert np.all(np.abs(got - ref) <= BWD_TOL * np.abs(ref))
