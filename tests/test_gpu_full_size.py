"""Parity at the full benchmark sizes, in the launch configuration bench.py times: whole (z, h) slices
for the smaller workloads, sampled output rows (computed one by one by the oracle's row evaluators) for
the largest ones, plus the properties that hold at any size (exact zeros in padding, determinism)."""
import numpy as np
import pytest

import oracle
from paper_2604_27124_amd import workloads as W
from gpu_util import BWD_TOL, FWD_TOL, Dev, check_against_oracle, slice_err, to_host

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def sampled_rows_check(w, dev, slices, rows_per_slice=24, seed=0):
    """Compare sampled rows of O, dQ, dK, dV with the oracle's row evaluators.  The norm's denominator
    (max |ref| of the slice) is taken over the sampled rows, which can only make the test stricter
    than the whole-slice norm by a small factor; the tolerance is unchanged."""
    rng = np.random.default_rng(seed)
    o = to_host(dev.fwd())
    dq, dk, dv = (to_host(t) for t in dev.bwd())
    worst = dict(o=0.0, dq=0.0, dk=0.0, dv=0.0)
    for z in range(w.B):
        n = int(w.seqlens[z])
        for a in (o, dq, dk, dv):
            assert np.all(a[z, n:] == 0.0)
    for z, h in slices:
        n = int(w.seqlens[z])
        rows = sorted(set([0, n - 1, n // 2] + rng.integers(0, n, rows_per_slice).tolist()))
        args = (w.q, w.k, w.v)
        ro = oracle.fwd_rows(*args, w.seqlens, w.bias, w.scale, z, h, rows)
        rq = oracle.bwd_q_rows(*args, w.d_o, w.seqlens, w.bias, w.scale, z, h, rows)
        rk, rv = oracle.bwd_kv_rows(*args, w.d_o, w.seqlens, w.bias, w.scale, z, h, rows)
        for key, got, ref, tol in (("o", o, ro, FWD_TOL), ("dq", dq, rq, BWD_TOL), ("dk", dk, rk, BWD_TOL),
                                   ("dv", dv, rv, BWD_TOL)):
            e = slice_err(got[z, rows, h], ref)
            worst[key] = max(worst[key], e)
            assert e <= tol, f"{key}: slice {(z, h)} n={n} sampled-row error {e:.3e} > {tol}"
    return worst


def test_unpadded_config_whole_slices():
    w = W.generate("unpadded", 0)
    say("unpadded", check_against_oracle(w, slices=[(0, 0), (3, 7), (7, 11)]))


def test_jagged_config():
    w = W.generate("jagged", 0)
    dev = Dev(w)
    order = np.argsort(w.seqlens)
    zs = [int(order[0]), int(order[-1]), int(order[len(order) // 2])]
    say("jagged lengths", w.seqlens.tolist())
    say("jagged whole slice (shortest)", check_against_oracle(w, slices=[(zs[0], 5)], dev=dev))
    say("jagged sampled", sampled_rows_check(w, dev, [(z, h) for z in range(w.B) for h in (z % w.H,)]))


def test_long_config_metric_point():
    # the metric point: three whole (z, h) slices of every sequence, sampled rows on three other heads of
    # every sequence, exact zeros in all padding, bitwise determinism
    w = W.generate("long", 0)
    dev = Dev(w)
    say("long lengths", w.seqlens.tolist())
    whole = [(z, h) for z in range(w.B) for h in (1, 6, 10)]
    say("long whole slices", whole, check_against_oracle(w, slices=whole, dev=dev))
    say("long sampled", sampled_rows_check(w, dev, [(z, h) for z in range(w.B) for h in (0, 5, 11)]))
    first = [to_host(dev.fwd())] + [to_host(t) for t in dev.bwd()]
    again = [to_host(dev.fwd())] + [to_host(t) for t in dev.bwd()]
    for x, y in zip(first, again):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("seed", [1, 2])
def test_long_config_other_seeds(seed):
    # the other two benchmarked draws of the lengths: one whole slice (shortest sequence) and sampled rows
    # on two heads of every sequence
    w = W.generate("long", seed)
    dev = Dev(w)
    say("long lengths", seed, w.seqlens.tolist())
    z = int(np.argmin(w.seqlens))
    say("long whole slice (shortest)", check_against_oracle(w, slices=[(z, 4)], dev=dev))
    say("long sampled", sampled_rows_check(w, dev, [(z, h) for z in range(w.B) for h in (2, 9)], seed=seed))


def test_wide_head_config():
    # d = 128 (dK / dV run as the role-swapped forward / dQ pair): one whole slice per sequence, sampled
    # rows on three more
    w = W.generate("wide", 0)
    dev = Dev(w)
    say("wide lengths", w.seqlens.tolist())
    say("wide whole slices", check_against_oracle(w, slices=[(0, 3), (1, 12)], dev=dev))
    say("wide sampled", sampled_rows_check(w, dev, [(0, 0), (1, 15), (0, 9)], rows_per_slice=16))


@pytest.mark.parametrize("cell", [dict(d=64, H=32, N=512, B=32, pad=0.25), dict(d=64, H=32, N=512, B=32, pad=0.0),
                                  dict(d=128, H=16, N=2048, B=8, pad=0.25)])
def test_paper_grid_cells(cell):
    # cells of the paper's kernel benchmark grid (Sec. 4 "Kernel performance": 16384 tokens per batch, hidden
    # size 2048, every sequence at (1 - pad) N valid tokens), as the sweep module launches them
    n = int(round(cell["N"] * (1.0 - cell["pad"])))
    w = W.make(cell["B"], cell["N"], cell["H"], cell["d"], (n,) * cell["B"], seed=77)
    slices = [(0, 0), (cell["B"] // 2, cell["H"] // 2), (cell["B"] - 1, cell["H"] - 1), (3, 1)]
    say("grid cell", cell, check_against_oracle(w, slices=slices))


def test_very_long_single_sequence_sampled_rows():
    # one sequence far beyond the benchmark lengths (625 streamed tiles, a ragged tail, 157 owner tiles):
    # exercises the 64-bit slice offsets and the longest streamed loop
    w = W.make(1, 40000, 2, 64, (39987,), seed=9)
    dev = Dev(w)
    say("N=40000 sampled", sampled_rows_check(w, dev, [(0, 0), (0, 1)], rows_per_slice=12))


def test_many_heads_wide_rows_sampled():
    # large row stride (H * d = 8192 elements): lane offsets inside a streamed tile stay 32-bit
    w = W.make(2, 1500, 64, 128, (1500, 700), seed=10)
    dev = Dev(w)
    say("H=64 d=128 sampled", sampled_rows_check(w, dev, [(0, 0), (1, 63), (0, 31)], rows_per_slice=8))
