"""GPU parity of the bias gradient (Sec. 3: learnable bias; db_z = sum over heads and valid pairs of dS)
and of the dQ that the same entry point returns, against the fp64 oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_27124_amd import binding
from paper_2604_27124_amd import workloads as W
from gpu_util import BWD_TOL, to_dev, to_host

pytestmark = pytest.mark.gpu


def run(w):
    q, k, v, g = to_dev(w.q), to_dev(w.k), to_dev(w.v), to_dev(w.d_o)
    s, b = torch.from_numpy(w.seqlens).cuda(), torch.from_numpy(w.bias).cuda()
    dq, db = binding.sigmoid_attn_bwd_dq_dbias(q, k, v, g, s, b, w.scale, dq=torch.full_like(q, float("nan")),
                                               dbias=torch.full((w.B,), float("nan"), device="cuda"))
    dq_only = binding.sigmoid_attn_bwd_dq(q, k, v, g, s, b, w.scale)
    dq2, db2 = binding.sigmoid_attn_bwd_dq_dbias(q, k, v, g, s, b, w.scale)
    torch.cuda.synchronize()
    assert torch.equal(dq.view(torch.int16), dq_only.view(torch.int16))        # same dQ as the plain kernel
    assert torch.equal(db, db2) and torch.equal(dq.view(torch.int16), dq2.view(torch.int16))   # reproducible
    _, _, _, ref = oracle.cross_bwd(w.q, w.k, w.v, w.d_o, w.seqlens, w.seqlens, w.bias, w.scale)
    return db.cpu().numpy().astype(np.float64), ref


def test_dbias_without_cancellation_d64():
    # dO >= 0 and V >= 0 make every dS non-negative, so the sum does not cancel and the relative error of
    # db is the relative error of its terms (bf16 dS, fp32 sums).
    w = W.make(3, 300, 2, 64, (300, 129, 0), seed=5)
    w.v[:] = np.abs(w.v); w.d_o[:] = np.abs(w.d_o)
    got, ref = run(w)
    print("dbias (positive terms)", got, ref, flush=True)
    assert got[2] == 0.0 and ref[2] == 0.0
    assert np.all(np.abs(got[:2] - ref[:2]) <= BWD_TOL * np.abs(ref[:2]))


@pytest.mark.parametrize("d", [64, 128])
def test_dbias_random_signs(d):
    # With random signs db is a sum of N = H n^2 terms of either sign; the natural scale of its error is
    # that of the terms, sqrt(sum dS^2), not |db|.  The bar: |error| <= 2e-2 * (|db| + sqrt(sum dS^2)).
    w = W.make(2, 200, 2, d, (200, 77), seed=6)
    got, ref = run(w)
    for z in range(2):
        ss = 0.0
        for h in range(w.H):
            _, _, ds = oracle.matrices(w.q, w.k, w.v, w.d_o, w.seqlens, w.bias, w.scale, z, h)
            ss += float(np.sum(ds * ds))
        bar = BWD_TOL * (abs(ref[z]) + np.sqrt(ss))
        print("dbias", d, z, got[z], ref[z], "bar", bar, flush=True)
        assert abs(got[z] - ref[z]) <= bar


def test_dbias_on_the_tiny_workload():
    w = W.generate("tiny", 0)
    got, ref = run(w)
    scale = np.abs(ref).max()
    assert np.all(np.abs(got - ref) <= BWD_TOL * scale + 1e-3)


@pytest.mark.parametrize("d", [64, 128])
def test_cross_dbias_with_separate_lengths(d):
    # queries and keys of different padded and valid lengths; V, dO >= 0 so that db does not cancel
    B, Lq, Lk, H = 3, 300, 520, 2
    rng = np.random.default_rng(40 + d)
    mk = lambda L: W.round_to_bf16(rng.standard_normal((B, L, H, d)).astype(np.float32))
    q, k, v, g = mk(Lq), mk(Lk), np.abs(mk(Lk)), np.abs(mk(Lq))
    nq, nk = np.array([300, 41, 0], np.int32), np.array([77, 520, 300], np.int32)
    bias = np.array([-4.0, -6.0, -5.0], np.float32)
    scale = 1.0 / np.sqrt(d)
    tq, tk, tv, tg = to_dev(q), to_dev(k), to_dev(v), to_dev(g)
    sq, sk, tb = torch.from_numpy(nq).cuda(), torch.from_numpy(nk).cuda(), torch.from_numpy(bias).cuda()
    dq, db = binding.sigmoid_attn_cross_bwd_dq_dbias(tq, tk, tv, tg, sq, sk, tb, scale,
                                                     dq=torch.full_like(tq, float("nan")),
                                                     dbias=torch.full((B,), float("nan"), device="cuda"))
    dq_ref, _, _ = binding.sigmoid_attn_cross_bwd(tq, tk, tv, tg, sq, sk, tb, scale)
    torch.cuda.synchronize()
    assert torch.equal(dq.view(torch.int16), dq_ref.view(torch.int16))      # same dQ as the plain cross kernel
    _, _, _, ref = oracle.cross_bwd(q, k, v, g, nq, nk, bias, scale)
    got = db.cpu().numpy().astype(np.float64)
    print("cross dbias", d, got, ref, flush=True)
    assert got[2] == 0.0 and ref[2] == 0.0                                  # no valid queries
    assert np.all(np.abs(got[:2] - ref[:2]) <= BWD_TOL * np.abs(ref[:2]))
