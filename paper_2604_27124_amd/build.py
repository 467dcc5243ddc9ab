"""Builds libsigattn.so (HIP, gfx950 only) in-tree with hipcc.  No JIT, no fallback."""
from __future__ import annotations

import os
import shutil
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libsigattn.so")
SOURCES = ["sigattn_api.hip"]
PROBE_LIB = os.path.join(HERE, "libmachine_probes.so")  # measurement aids for the benchmark, a library of their own
PROBE_SOURCES = ["machine_probes.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed-fp32 VALU forms are switched off for every device function of this library
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def hipcc() -> str:
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found: libsigattn needs the ROCm toolchain")
    return exe


def _compile(lib: str, sources, verbose: bool) -> str:
    cmd = [hipcc(), *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC, "-o", lib,
           *[os.path.join(CSRC, s) for s in sources]]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if verbose or res.returncode != 0:
        print(" ".join(cmd))
        print(res.stdout)
        print(res.stderr)
    if res.returncode != 0:
        raise RuntimeError(f"hipcc failed building {os.path.basename(lib)}")
    return lib


def build_library(verbose: bool = False) -> str:
    """libsigattn.so (the method) and libmachine_probes.so (the benchmark's measurement aids)."""
    _compile(PROBE_LIB, PROBE_SOURCES, verbose)
    return _compile(LIB, SOURCES, verbose)


if __name__ == "__main__":
    print(build_library(verbose=True))
