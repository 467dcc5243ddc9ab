"""GPU parity: the HIP path through the C ABI against the fp64 oracle, element by element, on the
same seeded inputs.  Tolerances: max |gpu - ref| / max |ref| per (z, h) slice <= 1e-2 for O and
<= 2e-2 for dQ, dK, dV (bf16 inputs); padded rows must be exact zeros."""
import numpy as np
import pytest
import torch

import oracle
from paper_2604_27124_amd import binding
from paper_2604_27124_amd import workloads as W
from gpu_util import (BWD_TOL, FWD_TOL, Dev, all_slices, check_against_oracle, check_slices, slice_err, to_dev,
                      to_host)

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def test_tiny_config_all_slices():
    w = W.generate("tiny", 0)
    say("tiny", w.seqlens, check_against_oracle(w))


@pytest.mark.parametrize("seqlens", [(0, 0), (1, 0), (300, 1), (63, 64), (65, 127), (128, 129), (255, 257),
                                     (300, 299), (31, 33)])
def test_edge_lengths_d64(seqlens):
    # N_max = 300 is not a multiple of any tile; lengths sit on and around tile edges
    w = W.make(2, 300, 2, 64, seqlens, seed=sum(seqlens) + 1)
    say("edge d64", seqlens, check_against_oracle(w))


@pytest.mark.parametrize("seqlens", [(0, 1), (130, 64), (200, 97)])
def test_edge_lengths_d128(seqlens):
    w = W.make(2, 200, 2, 128, seqlens, seed=sum(seqlens) + 2)
    say("edge d128", seqlens, check_against_oracle(w))


def test_several_tiles_ragged_tail_d64():
    w = W.make(3, 700, 3, 64, (700, 389, 513), seed=11)
    say("ragged d64", check_against_oracle(w))


def test_several_tiles_ragged_tail_d128():
    w = W.make(2, 520, 2, 128, (520, 263), seed=12)
    say("ragged d128", check_against_oracle(w))


@pytest.mark.parametrize("seed", range(10))
def test_random_shapes(seed):
    # shapes, lengths and head counts drawn at random (seeded): tile edges, owner blocks and the work
    # mapping are hit in combinations the hand-picked cases do not list
    rng = np.random.default_rng(1000 + seed)
    d = 64 if seed % 3 else 128
    B, H = int(rng.integers(1, 6)), int(rng.integers(1, 5))
    N = int(rng.integers(1, 641))
    seqlens = tuple(int(x) for x in rng.integers(0, N + 1, size=B))
    w = W.make(B, N, H, d, seqlens, seed=seed, qkv_std=float(rng.uniform(0.5, 2.0)))
    say("random shape", dict(B=B, N=N, H=H, d=d, seqlens=seqlens), check_against_oracle(w))


def test_large_logits_saturate_without_nan():
    w = W.make(1, 256, 2, 64, (200,), seed=13, qkv_std=4.0)      # |scale * s| up to ~ 60
    say("large logits", check_against_oracle(w))
    # one query row whose scores are exactly +-1024 (scale * s = +-128): 2^t' overflows to +inf for half of
    # its pairs (weight exactly 0) and underflows to 0 for the others (weight exactly 1); its neighbours in
    # the same tiles are ordinary pairs.  Nothing may turn into NaN (0 x inf), dQ of that row is ~ 0.
    w = W.make(1, 256, 2, 64, (200,), seed=16)
    sign = np.where(np.random.default_rng(16).random(256) < 0.5, -1.0, 1.0).astype(np.float32)
    w.q[0, 5] = 0.0
    w.q[0, 5, :, 0] = 32.0
    w.k[0, :, :, 0] = 32.0 * sign[:, None]
    say("overflowing exponentials", check_against_oracle(w))
    w = W.make(1, 256, 1, 64, (256,), seed=15, bias=[-200.0])    # weights underflow to 0
    dev = Dev(w)
    o = to_host(dev.fwd())
    assert np.all(np.isfinite(o)) and np.abs(o).max() < 1e-30
    for t in dev.bwd():
        assert np.all(np.isfinite(to_host(t)))


@pytest.mark.parametrize("bias", [4.0, 8.0, 12.0, 16.0, 20.0, 30.0, 60.0, -30.0])
def test_saturated_weights_keep_their_gradient(bias):
    # Weights close to 1 (score + bias >> 0): 1 - P falls below fp32 resolution next to 1, yet
    # dS = P (1 - P) dP (Alg. 2 / Alg. 3) stays a well-defined small number, which the oracle keeps through
    # sigma(x) sigma(-x).  All four tensors are compared with the oracle at every bias, under the parity norm.
    # The negative bias is the mirror case (weights close to 0).
    w = W.make(1, 256, 1, 64, (256,), seed=14, bias=[bias])
    say("bias", bias, check_against_oracle(w))


def test_padded_inputs_do_not_influence_valid_outputs():
    w = W.make(2, 320, 2, 64, (320, 150), seed=21)
    a = Dev(w)
    ref = [to_host(a.fwd())] + [to_host(t) for t in a.bwd()]
    w2 = W.make(2, 320, 2, 64, (320, 150), seed=21)
    rng = np.random.default_rng(5)
    for x in (w2.q, w2.k, w2.v, w2.d_o):                          # other finite data in the padded rows
        x[1, 150:] = W.round_to_bf16(100.0 * rng.standard_normal(x[1, 150:].shape).astype(np.float32))
    b = Dev(w2)
    new = [to_host(b.fwd())] + [to_host(t) for t in b.bwd()]
    for x, y in zip(ref, new):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("d", [64, 128])
def test_nan_and_inf_in_padded_rows_are_never_read(d):
    # Stronger than the contract (finite padding): padded streamed rows are never fetched (the loader
    # re-reads the last valid row and zeroes it) and padded owner rows are replaced by zeros at load, so
    # even NaN / Inf bit patterns in the padding leave every output bit unchanged.
    lens = (333, 150, 0)
    w = W.make(3, 333, 2, d, lens, seed=23)
    a = Dev(w)
    ref = [to_host(a.fwd())] + [to_host(t) for t in a.bwd()]
    w2 = W.make(3, 333, 2, d, lens, seed=23)
    bits = {"q": 0x7FC0, "k": 0x7F80, "v": 0xFF80, "d_o": 0xFFC1}      # NaN, +Inf, -Inf, another NaN
    b = Dev(w2)
    for nm, pat in bits.items():
        raw = getattr(b, nm).view(torch.int16)
        for z, n in enumerate(lens):
            raw[z, n:] = pat - 65536 if pat >= 32768 else pat
    torch.cuda.synchronize()
    new = [to_host(b.fwd())] + [to_host(t) for t in b.bwd()]
    for x, y in zip(ref, new):
        assert np.all(np.isfinite(y))
        assert np.array_equal(x, y)


# ---- the 512-row forward instance (two owner blocks per wave), selected when the key side is padded to
# more than 4096 rows: edge lengths, NaN padding, and agreement with the 256-row instance

WIDE_TILE_N = 4160          # just above 4096: the forward launch takes 512-row owner tiles


@pytest.mark.parametrize("seqlens", [(511, 512, 513, 4097), (544, 545, 32, 4160), (0, 1, 1025, 3000)])
def test_wide_forward_tile_edge_lengths(seqlens):
    # lengths on and around the 512-row owner tile, a wave whose second 32-row block is wholly padded
    # (544 = 512 + 32), a single valid row, an empty sequence, the full padded length
    w = W.make(4, WIDE_TILE_N, 2, 64, seqlens, seed=sum(seqlens) % 1000 + 3)
    say("512-row forward tile", seqlens, check_against_oracle(w, bwd=False))


def test_wide_forward_tile_nan_padding():
    lens = (513, 4097, 0)
    w = W.make(3, WIDE_TILE_N, 1, 64, lens, seed=91)
    ref = to_host(Dev(w).fwd())
    b = Dev(W.make(3, WIDE_TILE_N, 1, 64, lens, seed=91))
    for nm, pat in {"q": 0x7FC0, "k": 0x7F80, "v": 0xFF80}.items():
        raw = getattr(b, nm).view(torch.int16)
        for z, n in enumerate(lens):
            raw[z, n:] = pat - 65536 if pat >= 32768 else pat
    torch.cuda.synchronize()
    new = to_host(b.fwd())
    assert np.all(np.isfinite(new)) and np.array_equal(ref, new)


def test_forward_tile_shapes_agree():
    # the same sequences under N_max = 4096 (256-row owner tiles) and N_max = 4160 (512-row owner tiles):
    # both match the oracle, and they agree with each other under the parity norm (the order of the fp32
    # sums over key tiles is the same, so in fact bit for bit)
    lens = (4096, 1300, 513)
    a = W.make(3, 4096, 2, 64, lens, seed=92)
    b = W.make(3, WIDE_TILE_N, 2, 64, lens, seed=93)
    for nm in ("q", "k", "v", "d_o"):
        getattr(b, nm)[:, :4096] = getattr(a, nm)
    b.bias[:] = a.bias
    say("256-row tiles", check_against_oracle(a, bwd=False, slices=[(0, 0), (1, 1), (2, 0)]))
    say("512-row tiles", check_against_oracle(b, bwd=False, slices=[(0, 0), (1, 1), (2, 0)]))
    oa, ob = to_host(Dev(a).fwd()), to_host(Dev(b).fwd())
    for z, n in enumerate(lens):
        for h in range(2):
            assert slice_err(ob[z, :n, h], oa[z, :n, h].astype(np.float64)) < FWD_TOL
    say("tile shapes bitwise equal:", bool(np.array_equal(oa, ob[:, :4096])))


@pytest.mark.parametrize("B,N,H", [(300, 96, 1), (2000, 300, 2), (1100, 530, 1)])
def test_more_sequences_than_the_pairwise_ranking_holds(B, N, H):
    # B > 256: sequences are ranked by tile count with a histogram and block-wide prefix sums; every owner
    # tile of every (z, h) must still be produced exactly once (outputs are NaN-poisoned before the call,
    # so a tile that no workgroup took shows), and sampled slices must match the oracle.
    rng = np.random.default_rng(3 + B)
    lens = rng.integers(0, N + 1, size=B)
    lens[:4] = (N, 0, 1, 257 if N > 257 else N - 1)
    w = W.make(B, N, H, 64, lens, seed=24)
    zs = [0, 1, 2, 3, B // 3, B // 2, B - 1, int(np.argmax(lens[4:])) + 4]
    dev = Dev(w)
    say("large batch", (B, N, H), check_against_oracle(w, slices=[(z, z % H) for z in zs], dev=dev))
    for t in [dev.fwd()] + list(dev.bwd()):
        got = to_host(t)
        assert np.all(np.isfinite(got))
        for z in range(B):
            assert np.all(got[z, int(lens[z]):] == 0.0)
        nz = np.any(got != 0.0, axis=(2, 3))                  # [B, N]: rows that hold any non-zero value
        for z in (4, 5, B // 4, B - 2):
            assert nz[z, :int(lens[z])].all()                 # (random data: a valid row is never all zero)


def test_on_a_side_stream():
    w = W.make(2, 200, 2, 64, (200, 131), seed=25)
    q, k, v, g = (to_dev(x) for x in (w.q, w.k, w.v, w.d_o))
    sl, b = torch.from_numpy(w.seqlens).cuda(), torch.from_numpy(w.bias).cuda()
    ref_o = binding.sigmoid_attn_fwd(q, k, v, sl, b, w.scale)
    ref_g = binding.sigmoid_attn_bwd(q, k, v, g, sl, b, w.scale)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        o = binding.sigmoid_attn_fwd(q, k, v, sl, b, w.scale, stream=side)
        grads = binding.sigmoid_attn_bwd(q, k, v, g, sl, b, w.scale, stream=side)
    side.synchronize()
    assert torch.equal(o.view(torch.int16), ref_o.view(torch.int16))
    for x, y in zip(grads, ref_g):
        assert torch.equal(x.view(torch.int16), y.view(torch.int16))


def test_padding_invariance_across_n_max():
    # the same sequence under a larger N_max and with another batch neighbour: identical valid rows
    w = W.make(1, 200, 2, 64, (200,), seed=31)
    big = W.make(2, 448, 2, 64, (77, 200), seed=32)
    for nm in ("q", "k", "v", "d_o"):
        getattr(big, nm)[1, :200] = getattr(w, nm)[0]
    big.bias[1] = w.bias[0]
    a, b = Dev(w), Dev(big)
    ra = [to_host(a.fwd())] + [to_host(t) for t in a.bwd()]
    rb = [to_host(b.fwd())] + [to_host(t) for t in b.bwd()]
    for x, y in zip(ra, rb):
        assert np.array_equal(x[0], y[1, :200])


def test_run_to_run_determinism():
    w = W.make(2, 512, 2, 64, (512, 301), seed=41)
    dev = Dev(w)
    first = [to_host(dev.fwd())] + [to_host(t) for t in dev.bwd()]
    for _ in range(3):
        again = [to_host(dev.fwd())] + [to_host(t) for t in dev.bwd()]
        for x, y in zip(first, again):
            assert np.array_equal(x, y)


def test_inputs_are_not_modified():
    w = W.make(1, 256, 2, 64, (190,), seed=51)
    dev = Dev(w)
    dev.fwd(); dev.bwd()
    for t, ref in ((dev.q, w.q), (dev.k, w.k), (dev.v, w.v), (dev.d_o, w.d_o)):
        assert np.array_equal(to_host(t), ref)


def test_permutation_equivariance():
    w = W.make(1, 256, 1, 64, (180,), seed=61)
    base = Dev(w)
    o, (dq, dk, dv) = to_host(base.fwd()), [to_host(t) for t in base.bwd()]
    rng = np.random.default_rng(1)
    pq, pk = rng.permutation(180), rng.permutation(180)
    w2 = W.make(1, 256, 1, 64, (180,), seed=61)
    w2.q[0, :180] = w.q[0, pq]; w2.d_o[0, :180] = w.d_o[0, pq]
    w2.k[0, :180] = w.k[0, pk]; w2.v[0, :180] = w.v[0, pk]
    perm = Dev(w2)
    o2, (dq2, dk2, dv2) = to_host(perm.fwd()), [to_host(t) for t in perm.bwd()]
    # summation order changes, so compare under the parity norm (results of both runs are bf16)
    assert slice_err(o2[0, :180, 0], o[0, pq, 0].astype(np.float64)) < FWD_TOL
    assert slice_err(dq2[0, :180, 0], dq[0, pq, 0].astype(np.float64)) < BWD_TOL
    assert slice_err(dk2[0, :180, 0], dk[0, pk, 0].astype(np.float64)) < BWD_TOL
    assert slice_err(dv2[0, :180, 0], dv[0, pk, 0].astype(np.float64)) < BWD_TOL


def test_zero_query_closed_form_on_gpu():
    # Q = 0, b = -ln n: every weight is 1/(n+1), so O_i = sum_j v_j / (n+1)  (Sec. 3, b = -log n)
    w = W.make(1, 512, 2, 64, (400,), seed=71)
    w.q[:] = 0
    o = to_host(Dev(w).fwd())
    for h in range(2):
        ref = w.v[0, :400, h].astype(np.float64).sum(0) / 401.0
        assert slice_err(o[0, :400, h], np.broadcast_to(ref, (400, 64))) < FWD_TOL
