"""The entry point that allocates nothing (sigmoid_attn_bwd_dq_dbias_static: partial sums in the library's
own static device array) against the workspace form it is a variant of, through the C ABI: same dQ and
same db, bit for bit (same kernels, fixed summation order), on two calls in a row, the second on a
smaller input, so stale partials of the first call would show."""
import numpy as np
import pytest
import torch

from paper_2604_27124_amd import binding
from paper_2604_27124_amd import workloads as W
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def both(w):
    q, k, v, g = to_dev(w.q), to_dev(w.k), to_dev(w.v), to_dev(w.d_o)
    s, b = torch.from_numpy(w.seqlens).cuda(), torch.from_numpy(w.bias).cuda()
    ref_dq, ref_db = binding.sigmoid_attn_bwd_dq_dbias(q, k, v, g, s, b, w.scale)
    dq = torch.full_like(q, float("nan"))
    db = torch.full((w.B,), float("nan"), device="cuda", dtype=torch.float32)
    torch.cuda.synchronize()
    before = torch.cuda.memory_stats()["allocation.all.allocated"]
    binding.sigmoid_attn_bwd_dq_dbias_static(q, k, v, g, s, b, w.scale, dq=dq, dbias=db)
    after = torch.cuda.memory_stats()["allocation.all.allocated"]
    torch.cuda.synchronize()
    assert after == before                                   # the binding asked torch for nothing either
    assert torch.equal(dq.view(torch.int16), ref_dq.view(torch.int16))
    assert torch.equal(db.view(torch.int32), ref_db.view(torch.int32))
    assert bool(torch.isfinite(db).all())
    return db.cpu().numpy()


def test_static_scratch_matches_workspace_form_twice():
    big = W.make(3, 1000, 4, 64, (1000, 517, 0), seed=81)     # 48 query tiles
    small = W.make(2, 300, 2, 64, (150, 300), seed=82)        # 8 query tiles: reuses the front of the array
    first = both(big)
    second = both(small)
    print("db (static scratch)", first, second, flush=True)
    assert first[2] == 0.0
    wide = W.make(2, 260, 2, 128, (260, 131), seed=83)        # the d = 128 kernel
    both(wide)
