"""The library's calls only enqueue kernels (no allocation, no synchronisation, no memset), so a forward +
backward step can be captured into a HIP graph and replayed.  Every replay is compared with the eager
result, with eager work and synchronisations between the replays."""
import numpy as np
import pytest
import torch

from paper_2604_27124_amd import binding
from paper_2604_27124_amd import workloads as W
from gpu_util import to_dev

pytestmark = pytest.mark.gpu


def test_forward_backward_step_in_a_hip_graph():
    w = W.make(2, 700, 2, 64, (700, 431), seed=41)
    q, k, v, g = (to_dev(x) for x in (w.q, w.k, w.v, w.d_o))
    sl, b = torch.from_numpy(w.seqlens).cuda(), torch.from_numpy(w.bias).cuda()
    ws = torch.empty(max(binding.sigmoid_attn_bwd_dq_dbias_workspace_bytes(2, 700, 2, 64), 16), dtype=torch.uint8,
                     device="cuda")

    def step(o, dq, dk, dv, db, stream):
        binding.sigmoid_attn_fwd(q, k, v, sl, b, w.scale, out=o, stream=stream)
        binding.sigmoid_attn_bwd_dkdv(q, k, v, g, sl, b, w.scale, dk=dk, dv=dv, stream=stream)
        binding.sigmoid_attn_bwd_dq_dbias(q, k, v, g, sl, b, w.scale, dq=dq, dbias=db, workspace=ws, stream=stream)

    eager = [torch.empty_like(q) for _ in range(4)] + [torch.empty(2, device="cuda")]
    step(*eager, torch.cuda.current_stream())
    torch.cuda.synchronize()

    outs = [torch.empty_like(q) for _ in range(4)] + [torch.empty(2, device="cuda")]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step(*outs, side)                       # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step(*outs, torch.cuda.current_stream())
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()

    for replay in range(3):
        for t in outs:
            t.fill_(float("nan"))               # eager work between the replays (fill kernels, no memset)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for got, ref in zip(outs[:4], eager[:4]):
            assert torch.equal(got.view(torch.int16), ref.view(torch.int16)), f"replay {replay}"
        assert torch.equal(outs[4], eager[4]), f"replay {replay}"
