"""Pins for the oracle's stochastic rounding (Sec. 5.1: FP4 output gradients are rounded probabilistically to
the two nearest values).  The generator is pinned to the published known-answer vectors of Threefry-2x32-20
and to structural properties; the rounding to exact expectations obtained by enumerating all 256 random
bytes, to neighbour-only outputs and to its limits (RNE-independent scales, grid points fixed)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2602_01410_amd import workloads as wl

GRID = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


def test_threefry_known_answers():
    """The published known-answer vectors of Threefry-2x32 with 20 rounds (tests/golden/)."""
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "threefry2x32_20_kat.txt")
    rows = [[int(w, 16) for w in l.split()] for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for c0, c1, k0, k1, o0, o1 in rows:
        assert oracle.threefry2x32_20((c0, c1), (k0, k1)) == (o0, o1)


def test_threefry_is_a_bijection_of_the_counter_and_bytes_are_uniform():
    key = (0x1234, 0xABCD)
    outs = {oracle.threefry2x32_20((c, 7), key) for c in range(4096)}
    assert len(outs) == 4096                       # distinct counters -> distinct outputs (a keyed permutation)
    # byte stream: index -> byte; 2^16 bytes should fill all 256 values about evenly (chi-square, 255 dof)
    counts = np.bincount([oracle.sr_byte(99, i) for i in range(1 << 16)], minlength=256)
    chi2 = float(((counts - 256.0) ** 2 / 256.0).sum())
    assert 150.0 < chi2 < 380.0
    # different seeds give different streams, the same seed the same stream
    a = [oracle.sr_byte(1, i) for i in range(64)]
    assert a == [oracle.sr_byte(1, i) for i in range(64)]
    assert a != [oracle.sr_byte(2, i) for i in range(64)]


def test_sr_byte_layout():
    """Element j of a group of eight takes byte j of the generator's 64 bits (word 0 first, low byte first)."""
    seed = 0x0123456789ABCDEF
    for group in (0, 1, 5, (1 << 32) + 3):
        x0, x1 = oracle.threefry2x32_20((group & 0xFFFFFFFF, group >> 32), (seed & 0xFFFFFFFF, seed >> 32))
        want = [(x0 >> (8 * j)) & 255 for j in range(4)] + [(x1 >> (8 * j)) & 255 for j in range(4)]
        assert [oracle.sr_byte(seed, group * 8 + j) for j in range(8)] == want


def all_bf16_in(lo, hi):
    bits = np.arange(0x7F80, dtype=np.uint16)          # all finite non-negative bf16 values
    vals = wl.bf16_bits_to_f32(bits).astype(np.float64)
    return vals[(vals >= lo) & (vals <= hi)]


def test_sr_outputs_are_the_two_neighbours_and_grid_points_stay():
    for v in np.concatenate([all_bf16_in(2.0 ** -12, 6.0), [0.0]]):
        lo = max(g for g in GRID if g <= v)
        hi = min(g for g in GRID if g >= v)
        for sign in (1.0, -1.0):
            got = {oracle.decode(oracle.FP4, oracle.encode_sr_fp4(sign * v, r)) for r in (0, 1, 127, 128, 254, 255)}
            assert got <= {sign * lo, sign * hi}, (v, got)
            if lo == hi:
                assert got == {sign * lo}
    # the sign survives rounding to zero, as in the nearest-even path
    assert oracle.encode_sr_fp4(-1e-3, 255) == 8 and oracle.encode_sr_fp4(1e-3, 255) == 0
    # at or beyond the largest grid value: saturate
    assert oracle.encode_sr_fp4(7.0, 0) == 7 and oracle.encode_sr_fp4(-6.0, 255) == 15


def test_sr_expectation_is_exact_where_p_has_eight_bits():
    """Averaged over all 256 random bytes the rounded value equals v exactly for every bf16 magnitude in
    [0.25, 6] (there 256 p is an integer); below, the expectation is v rounded down to a multiple of
    0.5/256: never above v and less than 0.5/256 below it."""
    for v in all_bf16_in(0.25, 6.0):
        total = sum(Fraction(oracle.decode(oracle.FP4, oracle.encode_sr_fp4(v, r))) for r in range(256))
        assert total / 256 == Fraction(v), v
    step = Fraction(1, 512)
    for v in all_bf16_in(2.0 ** -14, 0.2499):
        total = sum(Fraction(oracle.decode(oracle.FP4, oracle.encode_sr_fp4(v, r))) for r in range(256))
        mean = total / 256
        assert mean <= Fraction(v) < mean + step, v
        assert mean == (Fraction(v) // step) * step


def test_sr_probability_is_monotone_in_the_random_byte():
    """up <=> rnd < threshold: once a value rounds down for some byte it rounds down for all larger bytes."""
    for v in (0.3, 0.77, 1.2, 1.7, 2.4, 3.9, 5.1):
        ups = [oracle.decode(oracle.FP4, oracle.encode_sr_fp4(v, r)) > v for r in range(256)]
        k = sum(ups)
        assert ups == [True] * k + [False] * (256 - k)


@pytest.mark.parametrize("axis", [oracle.ROW, oracle.COL])
def test_quantize_sr_scales_match_rne_and_codes_are_neighbours(axis):
    rng = np.random.default_rng(80 + axis)
    a = rng.standard_normal((64, 96)) * 10.0 ** rng.integers(-4, 4, size=(64, 1))
    a[3, :] = 0.0
    bits = wl.f32_to_bf16_bits(a.astype(np.float32))
    c_sr, s_sr = oracle.quantize_sr_fp4(bits, axis, oracle.NO_OVERFLOW, seed=5)
    c_ne, s_ne = oracle.quantize(bits, oracle.FP4, axis)
    assert np.array_equal(s_sr, s_ne)
    deq_sr = oracle.dequantize(c_sr, s_sr, oracle.FP4)
    deq_ne = oracle.dequantize(c_ne, s_ne, oracle.FP4)
    x = wl.bf16_bits_to_f32(bits).astype(np.float64)
    xs = x if axis == oracle.ROW else x.T
    # |sr - x| < one grid step at x's position: bounded by twice the nearest-even distance plus ... simpler:
    # both results bracket x or coincide with the nearest-even one
    same = deq_sr == deq_ne
    brackets = (np.minimum(deq_sr, deq_ne) <= xs) & (xs <= np.maximum(deq_sr, deq_ne))
    assert np.all(same | brackets)
    assert 0.05 < 1.0 - same.mean() < 0.6          # a fair share of elements does go the other way
    # another seed: same scales, different codes
    c2, s2 = oracle.quantize_sr_fp4(bits, axis, oracle.NO_OVERFLOW, seed=6)
    assert np.array_equal(s2, s_sr) and not np.array_equal(c2, c_sr)


def test_quantize_sr_mean_over_seeds_approaches_x():
    """Unbiasedness at tensor level: the average dequantized value over many seeds converges to x
    (elements above a quarter of their block's scaled range have exact expectation)."""
    rng = np.random.default_rng(82)
    bits = wl.f32_to_bf16_bits(rng.standard_normal((8, 64)).astype(np.float32))
    x = wl.bf16_bits_to_f32(bits).astype(np.float64)
    acc = np.zeros_like(x)
    n = 400
    for seed in range(n):
        c, s = oracle.quantize_sr_fp4(bits, oracle.ROW, oracle.NO_OVERFLOW, seed=seed)
        acc += oracle.dequantize(c, s, oracle.FP4)
    mean = acc / n
    scale = 2.0 ** (s.astype(np.float64) - 127.0).repeat(32, axis=1)
    # standard error of one element <= step/2/sqrt(n) with step <= 2 scaled units; allow 5 sigma + truncation bias
    assert np.all(np.abs(mean - x) <= scale * (5.0 * 1.0 / np.sqrt(n) + 1.0 / 256))
    # nearest-even is biased on this data by comparison: its error does not shrink
    c, s = oracle.quantize(bits, oracle.FP4, oracle.ROW)
    assert np.abs(oracle.dequantize(c, s, oracle.FP4) - x).mean() > 3 * np.abs(mean - x).mean()


def test_quantize_sr_element_uses_its_stored_index():
    """The byte an element gets depends on its position in the STORED matrix: quantizing the transpose along
    rows equals quantizing along columns."""
    rng = np.random.default_rng(83)
    bits = wl.f32_to_bf16_bits(rng.standard_normal((64, 32)).astype(np.float32))
    c1, s1 = oracle.quantize_sr_fp4(bits, oracle.COL, oracle.NO_OVERFLOW, seed=11)
    c2, s2 = oracle.quantize_sr_fp4(np.ascontiguousarray(bits.T), oracle.ROW, oracle.NO_OVERFLOW, seed=11)
    assert np.array_equal(c1, c2) and np.array_equal(s1, s2)
    # and element (r, c) really used byte number r * SC + c
    codes, scales = c2, s2
    xt = wl.bf16_bits_to_f32(np.ascontiguousarray(bits.T)).astype(np.float64)
    for (r, c) in ((0, 0), (5, 17), (31, 63)):
        sc = 2.0 ** (int(scales[r, c // 32]) - 127)
        want = oracle.encode_sr_fp4(xt[r, c] / sc, oracle.sr_byte(11, r * 64 + c))
        got = (int(codes[r, c // 2]) >> (4 * (c % 2))) & 15
        assert got == want
