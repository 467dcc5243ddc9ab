"""ctypes binding over libmfma_probe.so: the matrix-core ceiling the benchmark prints next to the
attention kernels.  A measurement aid in a library of its own; the method's library does not contain it."""
from __future__ import annotations

import ctypes
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmfma_probe.so")
EXPORTS = ("mfma_probe_operand_bytes", "mfma_probe_sink_bytes", "mfma_probe_flops", "mfma_probe_launch")

_lib = None


def load() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2604_27124_amd.build`")
        lib = ctypes.CDLL(LIB_PATH)
        lib.mfma_probe_operand_bytes.argtypes = []
        lib.mfma_probe_operand_bytes.restype = ctypes.c_size_t
        lib.mfma_probe_sink_bytes.argtypes = []
        lib.mfma_probe_sink_bytes.restype = ctypes.c_size_t
        lib.mfma_probe_flops.argtypes = [ctypes.c_int]
        lib.mfma_probe_flops.restype = ctypes.c_double
        lib.mfma_probe_launch.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p]
        lib.mfma_probe_launch.restype = ctypes.c_int
        _lib = lib
    return _lib


def tflops(kind: str = "random", iters: int = 20000, repeats: int = 3, stream=None) -> float:
    """Sustained rate (TFLOPS) of back-to-back bf16 MFMAs on `kind` operands ("random" N(0,1) or "constant"):
    the machine's matrix-core ceiling under this kind of data, measured with events on the launch stream."""
    import torch
    lib = load()
    n = lib.mfma_probe_operand_bytes() // 2
    if kind == "random":
        g = torch.Generator(device="cuda"); g.manual_seed(0)
        ops = torch.randn(n, device="cuda", generator=g).to(torch.bfloat16)
    elif kind == "constant":
        ops = torch.ones(n, device="cuda", dtype=torch.bfloat16)
    else:
        raise ValueError("kind must be 'random' or 'constant'")
    sink = torch.empty(lib.mfma_probe_sink_bytes() // 4, device="cuda", dtype=torch.float32)
    s = torch.cuda.current_stream() if stream is None else stream
    last = 0.0
    for _ in range(repeats):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(s)
        rc = lib.mfma_probe_launch(ops.data_ptr(), sink.data_ptr(), int(iters), int(s.cuda_stream))
        if rc != 0:
            raise RuntimeError(f"mfma_probe_launch failed with code {rc}")
        e1.record(s)
        e1.synchronize()
        last = lib.mfma_probe_flops(int(iters)) / (e0.elapsed_time(e1) * 1e-3) / 1e12   # the last repeat: clocks have settled
    return last
