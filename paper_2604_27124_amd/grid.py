"""Kernel benchmark grid in the paper's methodology (Sec. 4 "Kernel performance"; appendix "FLOP
Calculation"): sequence lengths 512 ... 16384 at a fixed 16384 tokens per batch, head dimension 64 and
128 at hidden size 2048 (32 / 16 heads), 0 % and 25 % padding, forward and backward timed separately,
about 100 ms of warm-up and then 250 timed iterations, mean and 99 % confidence interval, TFLOPS over
valid-token FLOPs.

    python -m paper_2604_27124_amd.grid [--iters 250] [--markdown out.md]

"25 % padding" is read as every sequence holding 0.75 N valid tokens (the paper does not say how it
pads).  Inputs are seeded synthetic bf16 normals drawn on the device; bias = -ln(valid length).
The paper's own numbers (H100, another machine) are not reproduced here; they are context only.
"""
from __future__ import annotations

import argparse
import json
import math
import sys


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=250)
    ap.add_argument("--warmup-ms", type=float, default=100.0)
    ap.add_argument("--tokens", type=int, default=16384)
    ap.add_argument("--markdown", default=None)
    args = ap.parse_args()

    import torch
    from . import binding

    if not torch.cuda.is_available():
        print("grid: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    binding.load()
    torch.manual_seed(0)
    stream = torch.cuda.current_stream()
    peak = 2516.6
    rows = []
    for d, H in ((64, 32), (128, 16)):
        for N in (512, 1024, 2048, 4096, 8192, 16384):
            B = args.tokens // N
            q, k, v, g = (torch.randn(B, N, H, d, device="cuda", dtype=torch.float32).to(torch.bfloat16)
                          for _ in range(4))
            o, dq, dk, dv = (torch.empty_like(q) for _ in range(4))
            for pad in (0.0, 0.25):
                n = int(round(N * (1.0 - pad)))
                seqlens = torch.full((B,), n, dtype=torch.int32, device="cuda")
                bias = torch.full((B,), -math.log(n), dtype=torch.float32, device="cuda")
                scale = 1.0 / math.sqrt(d)
                pairs = B * n * n
                flops = {"fwd": 4 * H * d * pairs, "bwd": 10 * H * d * pairs}

                def fwd():
                    binding.sigmoid_attn_fwd(q, k, v, seqlens, bias, scale, out=o, stream=stream)

                def bwd():
                    binding.sigmoid_attn_bwd(q, k, v, g, seqlens, bias, scale, dq=dq, dk=dk, dv=dv, stream=stream)

                for name, fn in (("fwd", fwd), ("bwd", bwd)):
                    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                    e0.record(stream)
                    spent = 0.0
                    while spent < args.warmup_ms:          # warm-up: at least warmup_ms of device time
                        for _ in range(10):
                            fn()
                        e1.record(stream)
                        e1.synchronize()
                        spent = e0.elapsed_time(e1)
                    evs = [torch.cuda.Event(enable_timing=True) for _ in range(args.iters + 1)]
                    evs[0].record(stream)
                    for i in range(args.iters):
                        fn()
                        evs[i + 1].record(stream)
                    torch.cuda.synchronize()
                    ms = torch.tensor([evs[i].elapsed_time(evs[i + 1]) for i in range(args.iters)], dtype=torch.float64)
                    mean = float(ms.mean())
                    ci = 2.576 * float(ms.std(unbiased=True)) / math.sqrt(args.iters)
                    tf = flops[name] / (mean * 1e-3) / 1e12
                    row = dict(d=d, H=H, N=N, B=B, padding=pad, valid=n, kernel=name, ms=round(mean, 5),
                               ci99_ms=round(ci, 5), tflops=round(tf, 1), pct_peak=round(100 * tf / peak, 2))
                    rows.append(row)
                    print(json.dumps(row), flush=True)
    if args.markdown:
        with open(args.markdown, "w") as f:
            f.write("| d | H | N | B | padding | fwd ms | fwd TFLOPS | bwd ms | bwd TFLOPS |\n|---|---|---|---|---|---|---|---|---|\n")
            for i in range(0, len(rows), 2):
                a, b = rows[i], rows[i + 1]
                f.write(f"| {a['d']} | {a['H']} | {a['N']} | {a['B']} | {int(a['padding'] * 100)} % | "
                        f"{a['ms']:.4f} ± {a['ci99_ms']:.4f} | {a['tflops']:.1f} | "
                        f"{b['ms']:.4f} ± {b['ci99_ms']:.4f} | {b['tflops']:.1f} |\n")
    return 0


if __name__ == "__main__":
    sys.exit(main())
