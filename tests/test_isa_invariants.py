"""Properties of the compiled gfx950 code that the kernels' synchronisation relies on, checked on the
assembly hipcc emits (cross-compiled here, no GPU needed).

The barrier that closes a streamed tile waits with `s_waitcnt lgkmcnt(k)` only until the tile's LDS
writes have completed, letting the k operand reads issued behind them stay in flight.  That is correct
only if (a) exactly k LDS reads, and nothing else that counts on that counter (no scalar loads), lie
between the writes and the barrier in the emitted code, and (b) the packed-fp32 forms stay switched off.
"""
import os
import re
import subprocess
import tempfile

import pytest

from paper_2604_27124_amd import build as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def kernels():
    """name -> list of instruction lines, one entry per kernel of the library."""
    with tempfile.TemporaryDirectory() as tmp:
        out = os.path.join(tmp, "api.s")
        flags = [f for f in B.HIPCC_FLAGS if f not in ("-shared", "-fPIC")]
        cmd = [B.hipcc(), *flags, "-I", os.path.join(ROOT, "include"), "-S", "--cuda-device-only", "-o", out,
               os.path.join(B.CSRC, "sigattn_api.hip")]
        subprocess.run(cmd, check=True, capture_output=True)
        text = open(out).read()
    result, name = {}, None
    for line in text.split("\n"):
        m = re.match(r"^(_ZN7sigattn14sigattn_kernel\w+):", line)
        if m:
            name = m.group(1)
            result[name] = {"body": [], "meta": {}}
            continue
        if name is None:
            continue
        m = re.match(r"^; (NumVgprs|ScratchSize|Occupancy): (\d+)", line)
        if m:
            result[name]["meta"][m.group(1)] = int(m.group(2))
        if line.startswith("\t.end_amdhsa_kernel") or line.startswith(".Lfunc_end"):
            pass
        ins = line.split(";")[0].strip()
        if ins and not ins.startswith("."):
            result[name]["body"].append(ins)
    assert len(result) >= 5
    return result


def mode_and_d(name):
    m = re.search(r"ILi(\d)ELi(\d+)E", name)
    return int(m.group(1)), int(m.group(2))


def test_tile_barrier_counts_its_reads(kernels):
    checked = 0
    for name, k in kernels.items():
        body = k["body"]
        for i, ins in enumerate(body):
            if ins != "s_barrier":
                continue
            # the LDS wait that belongs to the barrier: the nearest instruction before it that is not plain
            # ALU work (the compiler may slip a few such instructions in between; no LDS or scalar-memory
            # instruction may sit there)
            w = i - 1
            while w >= 0 and re.match(r"(v_|s_)(?!waitcnt|load|buffer_load|barrier)", body[w]) and i - w < 8:
                w -= 1
            m = re.match(r"s_waitcnt (?:vmcnt\(\d+\) )?lgkmcnt\((\d+)\)$", body[w])
            assert m, f"{name}: barrier without an LDS wait in front of it ({body[w]!r})"
            allowed = int(m.group(1))
            if allowed == 0:
                continue                      # a full wait is always safe
            assert w == i - 1, f"{name}: instructions between a partial LDS wait and its barrier"
            reads, j = 0, i - 2
            while j >= 0 and not body[j].startswith("ds_write"):
                assert not body[j].startswith(("s_load", "s_buffer_load", "s_barrier")), \
                    f"{name}: {body[j]!r} between the tile store and its barrier"
                if body[j].startswith("ds_read"):
                    reads += 1
                j -= 1
            assert j >= 0, f"{name}: partial LDS wait with no tile store before it"
            assert reads == allowed, f"{name}: lgkmcnt({allowed}) but {reads} LDS reads follow the tile store"
            checked += 1
    assert checked >= 4 * 5               # four unrolled ring slots in each of the five kernels


def test_no_packed_fp32_and_next_to_no_spills_at_d64(kernels):
    for name, k in kernels.items():
        for ins in k["body"]:
            assert not re.match(r"v_pk_(add|mul|fma)_f32", ins), f"{name}: packed fp32 instruction {ins!r}"
        mode, d = mode_and_d(name)
        if d == 64:
            # the 128-register forward instance (four waves per SIMD) may park two registers in scratch
            assert k["meta"].get("ScratchSize", 0) <= 16, f"{name}: register spills"
            assert k["meta"].get("NumVgprs", 0) <= 256


def test_hot_loops_use_the_matrix_and_transcendental_pipes(kernels):
    for name, k in kernels.items():
        ops = [ins.split()[0] for ins in k["body"]]
        assert ops.count("v_mfma_f32_32x32x16_bf16") > 64, name
        assert any(o.startswith("v_exp_f32") for o in ops) and any(o.startswith("v_rcp_f32") for o in ops), name
        assert any(o == "ds_read_b64_tr_b16" for o in ops), name
