"""The C-ABI library: it loads without a GPU, exports every symbol the header declares, and rejects
bad arguments on the host (before any HIP call), so all of this runs on the CPU."""
import ctypes
import os
import re

import pytest

from paper_2604_27124_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return B.load()


def test_exports_match_header(lib):
    header = open(os.path.join(ROOT, "include", "sigmoid_attn.h")).read()
    declared = set(re.findall(r"\b(sigmoid_attn_\w+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_benchmark_probe_library_is_separate_and_loads():
    """The matrix-core probe lives in a library and header of its own; the method's library has none of it."""
    from paper_2604_27124_amd import machine_probes as M
    header = open(os.path.join(ROOT, "paper_2604_27124_amd", "csrc", "machine_probes.h")).read()
    declared = set(re.findall(r"\b(machine_probe_\w+)\s*\(", header))
    assert declared == set(M.EXPORTS)
    probe = M.load()
    for name in declared:
        assert hasattr(probe, name), name
        assert not hasattr(B.load(), name)
    assert probe.machine_probe_mfma(None, None, 1, None) == -1          # rejected on the host
    assert probe.machine_probe_atomic(4096, 16, 1, 8, 1, None) == -1    # buffer too small
    assert probe.machine_probe_loop(4096, 1, 9, None) == -1             # no such component set
    assert probe.machine_probe_valu(4096, 1, 5, None) == -1             # no such arrangement
    assert probe.machine_probe_mfma_flops(1) == 512 * 8 * 32 * 2.0 * 32 * 32 * 16
    assert probe.machine_probe_atomic_updates(2, 3) == 2 * 4 * 3 * 32 * 64


def test_static_scratch_entry_point_rejects_on_the_host(lib):
    p = 4096                                                  # fake aligned device address: never dereferenced
    call = lambda **kw: lib.sigmoid_attn_bwd_dq_dbias_static(
        kw.get("q", p), p, p, kw.get("d_o", p), p, kw.get("dbias", p), p, p, 0.125,
        kw.get("B", 2), 256, 1, kw.get("d", 64), None)
    # 131072 query tiles fit the array (8 bytes each in 1 MiB); one more does not
    assert call(B=131073) == B.SIGATTN_ERR_TOO_LARGE
    assert call(d_o=None) == B.SIGATTN_ERR_INVALID_ARG
    assert call(q=p + 2) == B.SIGATTN_ERR_MISALIGNED
    assert call(dbias=p + 2) == B.SIGATTN_ERR_MISALIGNED
    assert call(d=96) == B.SIGATTN_ERR_UNSUPPORTED_D


def test_version_and_strerror(lib):
    assert B.sigmoid_attn_version() >= 100
    assert B.sigmoid_attn_strerror(0) == "success"
    texts = {B.sigmoid_attn_strerror(c) for c in range(-6, 1)}
    assert len(texts) == 7 and "unknown" in B.sigmoid_attn_strerror(-99)


def test_fwd_argument_validation(lib):
    p = 4096  # a fake, 16-byte aligned, never dereferenced device address
    ok = dict(B=2, N=256, H=2, d=64)

    def fwd(q=p, k=p, v=p, o=p, sl=p, b=p, scale=0.125, **kw):
        s = dict(ok); s.update(kw)
        return lib.sigmoid_attn_fwd(q, k, v, o, sl, b, scale, s["B"], s["N"], s["H"], s["d"], None)

    assert fwd(q=None) == B.SIGATTN_ERR_INVALID_ARG
    assert fwd(o=None) == B.SIGATTN_ERR_INVALID_ARG
    assert fwd(sl=None) == B.SIGATTN_ERR_INVALID_ARG
    assert fwd(b=None) == B.SIGATTN_ERR_INVALID_ARG
    assert fwd(B=0) == B.SIGATTN_ERR_INVALID_ARG
    assert fwd(N=-1) == B.SIGATTN_ERR_INVALID_ARG
    assert fwd(H=0) == B.SIGATTN_ERR_INVALID_ARG
    assert fwd(scale=float("nan")) == B.SIGATTN_ERR_INVALID_ARG
    assert fwd(scale=float("inf")) == B.SIGATTN_ERR_INVALID_ARG
    assert fwd(d=96) == B.SIGATTN_ERR_UNSUPPORTED_D
    assert fwd(d=32) == B.SIGATTN_ERR_UNSUPPORTED_D
    assert fwd(k=p + 8) == B.SIGATTN_ERR_MISALIGNED
    assert fwd(o=p + 2) == B.SIGATTN_ERR_MISALIGNED
    assert fwd(B=1 << 20, N=1 << 14, H=1) == B.SIGATTN_ERR_TOO_LARGE  # 2^40 elements per tensor
    # more than 256 sequences are ranked by tile count, in at most 1024 classes of 256 rows
    assert fwd(B=257, N=262145, H=1) == B.SIGATTN_ERR_TOO_LARGE


def test_bwd_argument_validation(lib):
    p = 4096

    def bwd(q=p, k=p, v=p, g=p, dq=p, dk=p, dv=p, sl=p, b=p, scale=0.125, Bn=2, N=256, H=2, d=64, ws=None, wsb=0):
        return lib.sigmoid_attn_bwd(q, k, v, g, dq, dk, dv, sl, b, scale, Bn, N, H, d, ws, wsb, None)

    assert bwd(g=None) == B.SIGATTN_ERR_INVALID_ARG
    assert bwd(dv=None) == B.SIGATTN_ERR_INVALID_ARG
    assert bwd(Bn=-3) == B.SIGATTN_ERR_INVALID_ARG
    assert bwd(d=80) == B.SIGATTN_ERR_UNSUPPORTED_D
    assert bwd(dq=p + 4) == B.SIGATTN_ERR_MISALIGNED
    assert bwd(g=p + 1) == B.SIGATTN_ERR_MISALIGNED
    need = B.sigmoid_attn_bwd_workspace_bytes(2, 256, 2, 64)
    if need > 0:
        assert bwd(ws=None, wsb=0) == B.SIGATTN_ERR_WORKSPACE
        assert bwd(ws=p, wsb=need - 1) == B.SIGATTN_ERR_WORKSPACE
    assert B.sigmoid_attn_bwd_workspace_bytes(0, 256, 2, 64) == 0
    assert B.sigmoid_attn_bwd_workspace_bytes(2, 256, 2, 96) == 0


def test_cross_argument_validation(lib):
    p = 4096

    def fwd(q=p, k=p, v=p, o=p, sq=p, sk=p, b=p, scale=0.125, Bn=2, Lq=128, Lk=300, H=2, d=64):
        return lib.sigmoid_attn_cross_fwd(q, k, v, o, sq, sk, b, scale, Bn, Lq, Lk, H, d, None)

    def bwd(q=p, k=p, v=p, g=p, dq=p, dk=p, dv=p, sq=p, sk=p, b=p, scale=0.125, Bn=2, Lq=128, Lk=300, H=2, d=128):
        return lib.sigmoid_attn_cross_bwd(q, k, v, g, dq, dk, dv, sq, sk, b, scale, Bn, Lq, Lk, H, d, None)

    assert fwd(sk=None) == B.SIGATTN_ERR_INVALID_ARG
    assert fwd(Lk=0) == B.SIGATTN_ERR_INVALID_ARG
    assert fwd(Lq=-1) == B.SIGATTN_ERR_INVALID_ARG
    assert fwd(d=32) == B.SIGATTN_ERR_UNSUPPORTED_D
    assert fwd(o=p + 8) == B.SIGATTN_ERR_MISALIGNED
    assert fwd(scale=float("inf")) == B.SIGATTN_ERR_INVALID_ARG
    assert fwd(H=1 << 15, d=128) == B.SIGATTN_ERR_TOO_LARGE
    assert bwd(sq=None) == B.SIGATTN_ERR_INVALID_ARG
    assert bwd(dk=None) == B.SIGATTN_ERR_INVALID_ARG
    assert bwd(Lk=0) == B.SIGATTN_ERR_INVALID_ARG
    assert bwd(dv=p + 2) == B.SIGATTN_ERR_MISALIGNED


def test_dq_dbias_argument_validation(lib):
    p = 4096
    need = B.sigmoid_attn_bwd_dq_dbias_workspace_bytes(2, 300, 3, 64)
    assert need == 2 * 3 * 2 * 8          # one (float, int32) pair per 256-row query tile of every (z, h)
    assert B.sigmoid_attn_bwd_dq_dbias_workspace_bytes(2, 300, 3, 100) == 0

    def f(q=p, g=p, dq=p, db=p, ws=p, wsb=need, d=64, Bn=2):
        return lib.sigmoid_attn_bwd_dq_dbias(q, p, p, g, dq, db, p, p, 0.125, Bn, 300, 3, d, ws, wsb, None)

    assert f(db=None) == B.SIGATTN_ERR_INVALID_ARG
    assert f(g=None) == B.SIGATTN_ERR_INVALID_ARG
    assert f(Bn=0) == B.SIGATTN_ERR_INVALID_ARG
    assert f(d=96) == B.SIGATTN_ERR_UNSUPPORTED_D
    assert f(dq=p + 2) == B.SIGATTN_ERR_MISALIGNED
    assert f(ws=None) == B.SIGATTN_ERR_WORKSPACE
    assert f(wsb=need - 1) == B.SIGATTN_ERR_WORKSPACE
    assert f(ws=p + 4) == B.SIGATTN_ERR_MISALIGNED
    assert f(db=p + 2) == B.SIGATTN_ERR_MISALIGNED


def test_cross_dq_dbias_argument_validation(lib):
    ok = ctypes.c_void_p(256)
    f = lib.sigmoid_attn_cross_bwd_dq_dbias
    args = lambda **kw: [kw.get(n, ok) for n in ("q", "k", "v", "d_o", "dq", "dbias", "sq", "sk", "bias")] + \
        [ctypes.c_float(kw.get("scale", 0.125)), kw.get("B", 2), kw.get("Lq", 300), kw.get("Lk", 520), kw.get("H", 2),
         kw.get("d", 64), kw.get("ws", ok), ctypes.c_size_t(kw.get("wsb", 1 << 20)), None]
    assert f(*args(sk=None)) == -1                       # a null pointer
    assert f(*args(Lk=0)) == -1                          # a non-positive size
    assert f(*args(d=96)) == -2                          # unsupported head dimension
    assert f(*args(k=ctypes.c_void_p(8))) == -3          # misaligned tensor
    assert f(*args(wsb=8)) == -4                         # workspace too small
    need = lib.sigmoid_attn_cross_bwd_dq_dbias_workspace_bytes(2, 300, 520, 2, 64)
    assert need == 2 * 2 * 2 * 8 == lib.sigmoid_attn_bwd_dq_dbias_workspace_bytes(2, 300, 2, 64)
    assert lib.sigmoid_attn_cross_bwd_dq_dbias_workspace_bytes(2, 300, 0, 2, 64) == 0


def test_binding_refuses_cpu_tensors():
    import torch
    x = torch.zeros(1, 8, 1, 64, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        B.sigmoid_attn_fwd(x, x, x, torch.zeros(1, dtype=torch.int32), torch.zeros(1), 0.125)


def test_header_is_plain_c_and_links_from_c(tmp_path):
    """The boundary is usable from C: the header compiles as C99 with warnings as errors, and a C
    program linked against the library reaches the host-only entry points (no GPU call is made)."""
    import subprocess
    src = tmp_path / "use_abi.c"
    src.write_text(
        '#include "sigmoid_attn.h"\n'
        '#include <stdio.h>\n'
        '#include <string.h>\n'
        'int main(void) {\n'
        '    if (sigmoid_attn_version() < 100) return 1;\n'
        '    if (strcmp(sigmoid_attn_strerror(0), "success") != 0) return 2;\n'
        '    if (sigmoid_attn_bwd_workspace_bytes(4, 8192, 12, 64) != 0) return 3;\n'
        '    /* null tensors: rejected on the host before any device work */\n'
        '    if (sigmoid_attn_fwd(NULL, NULL, NULL, NULL, NULL, NULL, 0.125f, 1, 64, 1, 64, NULL) >= 0) return 4;\n'
        '    puts("ok");\n'
        '    return 0;\n'
        '}\n')
    exe = tmp_path / "use_abi"
    libdir = os.path.dirname(B.LIB_PATH)
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-l:" + os.path.basename(B.LIB_PATH),
                    "-Wl,-rpath," + libdir], check=True, capture_output=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True)
    assert out.stdout.strip() == "ok"
