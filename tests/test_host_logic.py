"""Host-side behaviour of the benchmark and of the entry module that needs no GPU: the one-GPU rule,
loud failure without a device (there is no CPU fallback), and the shape of the oracle-timed baseline."""
import importlib.util
import os
import subprocess
import sys

import pytest
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def run(*args):
    return subprocess.run([sys.executable, *args], cwd=ROOT, capture_output=True, text=True, timeout=300)


def load_bench():
    spec = importlib.util.spec_from_file_location("bench_module", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_bench_refuses_more_than_one_gpu():
    r = run("bench.py", "--gpus", "2")
    assert r.returncode != 0 and r.stdout.strip() == ""
    assert "ONE GPU" in r.stderr


@pytest.mark.skipif(torch.cuda.is_available(), reason="checks the behaviour on a machine without a GPU")
def test_bench_and_grid_fail_loudly_without_a_gpu():
    for cmd in (("bench.py",), ("-m", "paper_2604_27124_amd.grid")):
        r = run(*cmd)
        assert r.returncode != 0 and r.stdout.strip() == ""
        assert "no CPU fallback" in r.stderr


def test_cpu_baseline_fields_and_flop_accounting():
    from paper_2604_27124_amd import workloads as W
    bench = load_bench()
    w = W.generate("tiny", 0)
    b = bench.cpu_baseline(w, budget_s=5.0)
    assert b["kind"] == "oracle" and b["unit"] == "TFLOPS" and b["cores"] >= 1 and b["value"] > 0
    assert "tiny" in b["sample"] and "4 of 4" in b["sample"]            # B = 2, H = 2: every slice fits the budget
    flops = 14 * w.d * w.H * sum(int(n) ** 2 for n in w.seqlens)
    assert abs(b["value"] * 1e12 * b["seconds"] - flops) <= 1e-6 * flops


def test_entry_module_exposes_build_and_smoke():
    spec = importlib.util.spec_from_file_location("graft_entry", os.path.join(ROOT, "__graft_entry__.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    assert callable(mod.build) and callable(mod.smoke)


def test_traffic_lookup_and_confidence_interval():
    import numpy as np
    bench = load_bench()
    # the tracked counter summary is keyed by workload, seed and kernel; anything else has no measurement
    t = bench.measured_traffic_bytes("long", 0, "bwd_dkdv")
    assert isinstance(t, int) and 1e8 < t < 1e9
    assert bench.measured_traffic_bytes("long", 1, "bwd_dkdv") is None
    assert bench.measured_traffic_bytes("tiny", 0, "fwd") is None
    m, h = bench.mean_ci99(np.array([1.0, 2.0, 3.0, 4.0]))
    assert m == 2.5 and abs(h - 2.576 * np.std([1, 2, 3, 4], ddof=1) / 2.0) < 1e-12
    assert bench.mean_ci99(np.array([5.0])) == (5.0, 0.0)
