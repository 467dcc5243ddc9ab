"""The seeded input generator: determinism, bf16 rounding, shapes and length rules."""
import math

import numpy as np

from paper_2604_27124_amd import workloads as W


def test_round_to_bf16_ties_to_even():
    x = np.array([1.0, 1.0 + 2 ** -8, 1.0 + 3 * 2 ** -8, 1.0 + 2 ** -8 + 2 ** -20, -1.0 - 2 ** -8, 0.0, 3.0e38],
                 np.float32)
    r = W.round_to_bf16(x)
    assert list(r[:6]) == [1.0, 1.0, 1.0 + 2 ** -6, 1.0 + 2 ** -7, -1.0, 0.0]
    assert np.isfinite(r[6])
    assert np.array_equal(W.bits_to_f32(W.bf16_bits(r)), r)
    assert W.bf16_bits(np.array([1.0, -2.0], np.float32)).tolist() == [0x3F80, 0xC000]


def test_generate_is_deterministic_and_shaped():
    a, b = W.generate("tiny", 0), W.generate("tiny", 0)
    assert a.seqlens.tolist() == [256, 173] and a.q.shape == (2, 256, 2, 64)
    for n in ("q", "k", "v", "d_o"):
        assert np.array_equal(getattr(a, n), getattr(b, n))
        assert np.array_equal(W.round_to_bf16(getattr(a, n)), getattr(a, n))
    c = W.generate("tiny", 1)
    assert not np.array_equal(a.q, c.q)
    assert a.scale == 1 / 8 and np.allclose(a.bias, [-math.log(256), -math.log(173)])
    assert np.all(np.isfinite(a.q[1, 173:]))                  # padded rows hold finite random data


def test_length_rules():
    rng = np.random.default_rng(0)
    n = W.draw_lengths(("lognormal", 1500.0, 0.8, 64, 4096), 4000, 4096, rng)
    assert n.min() >= 64 and n.max() == 4096 and 1350 < np.median(n) < 1650
    n = W.draw_lengths(("uniform", 1024, 8192), 4000, 8192, rng)
    assert n.min() >= 1024 and n.max() <= 8192 and 4300 < n.mean() < 4900
    assert W.draw_lengths(("full",), 3, 77, rng).tolist() == [77, 77, 77]
    assert W.default_bias(np.array([0, 1, 8])).tolist() == [0.0, 0.0, np.float32(-math.log(8))]
