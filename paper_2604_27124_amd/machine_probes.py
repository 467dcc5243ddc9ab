"""ctypes binding over libmachine_probes.so and a small driver: measurements of the machine that the
design of the attention kernels rests on (matrix-core ceiling, atomic-add rate, a model of the dK/dV
loop with removable components).  Measurement aids in a library of their own; the method's library
does not contain them.

    python -m paper_2604_27124_amd.machine_probes            # prints one JSON object per probe
"""
from __future__ import annotations

import ctypes
import json
import os
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmachine_probes.so")
EXPORTS = ("machine_probe_mfma_operand_bytes", "machine_probe_sink_bytes", "machine_probe_mfma_flops",
           "machine_probe_mfma", "machine_probe_atomic_bytes", "machine_probe_atomic_updates",
           "machine_probe_atomic", "machine_probe_loop_wave_slots_per_simd", "machine_probe_loop",
           "machine_probe_valu")

_lib = None


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_27124_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        vp, ci, sz, db = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t, ctypes.c_double
        lib.machine_probe_mfma_operand_bytes.argtypes = []
        lib.machine_probe_mfma_operand_bytes.restype = sz
        lib.machine_probe_sink_bytes.argtypes = []
        lib.machine_probe_sink_bytes.restype = sz
        lib.machine_probe_mfma_flops.argtypes = [ci]
        lib.machine_probe_mfma_flops.restype = db
        lib.machine_probe_mfma.argtypes = [vp, vp, ci, vp]
        lib.machine_probe_mfma.restype = ci
        lib.machine_probe_atomic_bytes.argtypes = []
        lib.machine_probe_atomic_bytes.restype = sz
        lib.machine_probe_atomic_updates.argtypes = [ci, ci]
        lib.machine_probe_atomic_updates.restype = db
        lib.machine_probe_atomic.argtypes = [vp, sz, ci, ci, ci, vp]
        lib.machine_probe_atomic.restype = ci
        lib.machine_probe_loop_wave_slots_per_simd.argtypes = [ci]
        lib.machine_probe_loop_wave_slots_per_simd.restype = db
        lib.machine_probe_loop.argtypes = [vp, ci, ci, vp]
        lib.machine_probe_loop.restype = ci
        lib.machine_probe_valu.argtypes = [vp, ci, ci, vp]
        lib.machine_probe_valu.restype = ci
        _lib = lib
    return _lib


def _timed(launch, repeats: int = 3) -> float:
    """Milliseconds of the last of `repeats` launches (clocks have settled by then), events on the current stream."""
    import torch
    s = torch.cuda.current_stream()
    ms = 0.0
    for _ in range(repeats):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(s)
        rc = launch(int(s.cuda_stream))
        if rc != 0:
            raise RuntimeError(f"machine probe failed with code {rc}")
        e1.record(s)
        e1.synchronize()
        ms = e0.elapsed_time(e1)
    return ms


def mfma_tflops(kind: str = "random", iters: int = 20000, repeats: int = 3) -> float:
    """Sustained rate (TFLOPS) of back-to-back bf16 MFMAs on `kind` operands ("random" N(0,1) or "constant")."""
    import torch
    lib = load()
    n = lib.machine_probe_mfma_operand_bytes() // 2
    if kind == "random":
        g = torch.Generator(device="cuda"); g.manual_seed(0)
        ops = torch.randn(n, device="cuda", generator=g).to(torch.bfloat16)
    elif kind == "constant":
        ops = torch.ones(n, device="cuda", dtype=torch.bfloat16)
    else:
        raise ValueError("kind must be 'random' or 'constant'")
    sink = torch.empty(lib.machine_probe_sink_bytes() // 4, device="cuda", dtype=torch.float32)
    ms = _timed(lambda st: lib.machine_probe_mfma(ops.data_ptr(), sink.data_ptr(), int(iters), st), repeats)
    return lib.machine_probe_mfma_flops(int(iters)) / (ms * 1e-3) / 1e12


def atomic_rate(atomic: bool, blocks: int = 2048, iters: int = 200) -> dict:
    """Giga 4-byte updates per second of fp32 atomic adds (or plain stores) in the dQ-flush pattern."""
    import torch
    lib = load()
    buf = torch.zeros(lib.machine_probe_atomic_bytes() // 4, device="cuda", dtype=torch.float32)
    ms = _timed(lambda st: lib.machine_probe_atomic(buf.data_ptr(), buf.numel() * 4, int(atomic), blocks, iters, st))
    n = lib.machine_probe_atomic_updates(blocks, iters)
    return {"kind": "atomic add" if atomic else "plain store", "blocks": blocks, "iters": iters, "ms": round(ms, 3),
            "giga_updates_per_s": round(n / (ms * 1e-3) / 1e9, 1), "TB_per_s": round(4 * n / (ms * 1e-3) / 1e12, 2)}


LOOP_COMPONENTS = {1: "VALU", 2: "LDS reads", 4: "MFMA"}


def loop_model(components: int, iters: int = 5000) -> dict:
    """SIMD time per wave-slot (ns) of the dK/dV loop model with the given components (bit 0 VALU, 1 LDS, 2 MFMA)."""
    import torch
    lib = load()
    sink = torch.empty(lib.machine_probe_sink_bytes() // 4, device="cuda", dtype=torch.float32)
    ms = _timed(lambda st: lib.machine_probe_loop(sink.data_ptr(), iters, components, st))
    names = [n for b, n in LOOP_COMPONENTS.items() if components & b] or ["barrier only"]
    if components == 8:
        names = ["VALU", "LDS reads", "two 16x16x32 MFMAs per slot"]
    return {"components": " + ".join(names), "ms": round(ms, 3),
            "ns_per_wave_slot": round(ms * 1e6 / lib.machine_probe_loop_wave_slots_per_simd(iters), 2)}


VALU_ARRANGEMENTS = ("as the kernels issue them (exp exp | fma fma rcp rcp | rest)", "all transcendentals in one run",
                     "single transcendentals evenly spread", "the 22 plain instructions only",
                     "the 8 transcendentals only")


def valu_mix(arrangement: int, iters: int = 40000) -> dict:
    """SIMD time (ns) per score element of the backward's vector work in the given arrangement."""
    import torch
    lib = load()
    sink = torch.empty(lib.machine_probe_sink_bytes() // 4, device="cuda", dtype=torch.float32)
    ms = _timed(lambda st: lib.machine_probe_valu(sink.data_ptr(), iters, arrangement, st))
    return {"arrangement": VALU_ARRANGEMENTS[arrangement], "ms": round(ms, 3),
            "ns_per_element": round(ms * 1e6 / iters / 2 / 4, 2)}      # two waves per SIMD, four elements per iteration


def tail_fill(workload: str, seed: int, steps: int = 60) -> dict:
    """ms per fwd+bwd step of a workload with the three kernels on one stream, with the two backward kernels
    on two streams, and with all three concurrent: does filling one kernel's schedule tail with another pay?"""
    import time
    import numpy as np
    import torch
    from . import binding
    from . import workloads as W
    w = W.generate(workload, seed)
    dev = lambda a: torch.from_numpy(W.bf16_bits(a).view(np.int16)).cuda().view(torch.bfloat16)
    q, k, v, g = dev(w.q), dev(w.k), dev(w.v), dev(w.d_o)
    sl, b = torch.from_numpy(w.seqlens).cuda(), torch.from_numpy(w.bias).cuda()
    o, dq, dk, dv = (torch.empty_like(q) for _ in range(4))
    s0, s1, s2 = torch.cuda.current_stream(), torch.cuda.Stream(), torch.cuda.Stream()
    fwd = lambda s: binding.sigmoid_attn_fwd(q, k, v, sl, b, w.scale, out=o, stream=s)
    dkdv = lambda s: binding.sigmoid_attn_bwd_dkdv(q, k, v, g, sl, b, w.scale, dk=dk, dv=dv, stream=s)
    dqk = lambda s: binding.sigmoid_attn_bwd_dq(q, k, v, g, sl, b, w.scale, dq=dq, stream=s)

    def fork(streams):
        e = torch.cuda.Event(); e.record(s0)
        for s in streams:
            s.wait_event(e)

    def join(streams):
        for s in streams:
            e = torch.cuda.Event(); e.record(s); s0.wait_event(e)

    def one(): fwd(s0); dkdv(s0); dqk(s0)
    def two(): fwd(s0); fork([s1]); dkdv(s0); dqk(s1); join([s1])
    def three(): fork([s1, s2]); dkdv(s0); dqk(s1); fwd(s2); join([s1, s2])

    out = {"workload": f"{workload} seed {seed}", "seqlens": [int(x) for x in w.seqlens]}
    for name, fn in (("one_stream_ms", one), ("bwd_on_two_streams_ms", two), ("all_three_concurrent_ms", three)):
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            fn()
        torch.cuda.synchronize()
        out[name] = round((time.perf_counter() - t0) / steps * 1e3, 4)
    return out


def main() -> int:
    import torch
    if not torch.cuda.is_available():
        print("machine_probes: no GPU visible", file=sys.stderr)
        return 2
    print(json.dumps({"probe": "mfma", "random_operands_tflops": round(mfma_tflops("random"), 1),
                      "constant_operands_tflops": round(mfma_tflops("constant"), 1)}), flush=True)
    for atomic in (True, False):
        print(json.dumps({"probe": "atomic", **atomic_rate(atomic)}), flush=True)
    for comp in (7, 8, 6, 5, 3, 4, 1, 2):
        print(json.dumps({"probe": "loop", **loop_model(comp)}), flush=True)
    for arr in range(5):
        print(json.dumps({"probe": "valu", **valu_mix(arr)}), flush=True)
    for wl, seed in (("long", 0), ("long", 2), ("long_full", 0)):
        print(json.dumps({"probe": "tail_fill", **tail_fill(wl, seed)}), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
