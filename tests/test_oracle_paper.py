"""Pins for the oracle's implementation of the paper's own recipe (Sec. 2.3: scale = FPX_MAX / max|x|,
cast, divide back; Sec. 5.1: 1x128 tiles for activations and gradients, 128x128 blocks for weights)."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_2602_01410_amd import workloads as wl

MAXV = {oracle.FP8: 448.0, oracle.FP4: 6.0}


def grid(fmt):
    n = 256 if fmt == oracle.FP8 else 16
    vals = [oracle.decode(fmt, c) for c in range(n)]
    return [(c, v) for c, v in enumerate(vals) if v == v]          # drop NaN codes


def nearest_code_exact(fmt, t: float) -> int:
    """Brute force on exact rationals: nearest grid value, ties to the even code, sign of t kept."""
    g = [(c, Fraction(v)) for c, v in grid(fmt) if (c < (128 if fmt == oracle.FP8 else 8))]
    a = abs(Fraction(t))
    best = min(g, key=lambda cv: (abs(cv[1] - a), cv[0] & 1))
    sign = (128 if fmt == oracle.FP8 else 8) if np.signbit(t) else 0
    return best[0] | sign


def bits_of(a):
    return wl.f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


@pytest.mark.parametrize("fmt", [oracle.FP8, oracle.FP4])
@pytest.mark.parametrize("group", [oracle.TILE_1x128, oracle.BLOCK_128x128])
def test_scales_are_fp32_quotients_and_codes_nearest(fmt, group):
    rng = np.random.default_rng(120 + fmt)
    a = rng.standard_normal((256, 256)) * 10.0 ** rng.integers(-3, 3, size=(256, 1))
    bits = bits_of(a)
    x = wl.bf16_bits_to_f32(bits)
    codes, scales = oracle.quantize_paper(bits, fmt, oracle.ROW, group)
    # scale: numpy's own float32 division of the type's maximum by the group maximum
    amax = np.abs(x).reshape(256 // group, group, 2, 128).max(axis=(1, 3))
    want_s = (np.float32(MAXV[fmt]) / amax.astype(np.float32)).astype(np.float32)
    assert np.array_equal(scales, want_s)
    # codes: numpy's float32 product, then an exact-rational nearest-value search, on a sample
    for _ in range(400):
        r, c = int(rng.integers(256)), int(rng.integers(256))
        t = np.float32(x[r, c]) * scales[r // group, c // 128]
        got = int(codes[r, c]) if fmt == oracle.FP8 else (int(codes[r, c // 2]) >> (4 * (c % 2))) & 15
        assert got == nearest_code_exact(fmt, float(t)), (r, c)
    # the group maximum lands on the largest code
    if fmt == oracle.FP8:
        mag = codes & 0x7F
    else:
        mag = np.stack([codes & 7, (codes >> 4) & 7], axis=-1).reshape(256, 256)
    top = mag.reshape(256 // group, group, 2, 128).max(axis=(1, 3))
    assert np.all(top == (0x7E if fmt == oracle.FP8 else 7))


@pytest.mark.parametrize("fmt", [oracle.FP8, oracle.FP4])
def test_representable_tiles_round_trip_exactly(fmt):
    """Grid values times a power of two, with the type's maximum present in every tile: the scale is a power
    of two, nothing rounds, the error statistics are zero."""
    rng = np.random.default_rng(122)
    vals = np.array(sorted({abs(v) for _, v in grid(fmt) if abs(v) * 128 == int(abs(v) * 128) and abs(v) >= 2.0 ** -6}))
    a = rng.choice(vals, size=(64, 256)) * rng.choice([-1.0, 1.0], size=(64, 256))
    a[:, 0] = MAXV[fmt]; a[:, 128] = -MAXV[fmt]
    a *= 2.0 ** rng.integers(-10, 10, size=(64, 1))
    bits = bits_of(a)
    assert np.array_equal(wl.bf16_bits_to_f32(bits).astype(np.float64), a)      # all exactly bf16
    codes, scales = oracle.quantize_paper(bits, fmt, oracle.ROW, oracle.TILE_1x128)
    assert np.array_equal(oracle.dequantize_paper(codes, scales, fmt, oracle.TILE_1x128), a)
    st = oracle.stats_paper(bits, oracle.ROW, oracle.TILE_1x128)
    assert np.isclose(st[0], (a ** 2).sum(), rtol=1e-13) and st[1 if fmt == oracle.FP4 else 2] == 0.0


def test_axis_is_transpose_and_blocks_of_equal_rows_are_tiles():
    rng = np.random.default_rng(123)
    bits = bits_of(rng.standard_normal((128, 256)))
    for fmt in (oracle.FP8, oracle.FP4):
        for group in (oracle.TILE_1x128, oracle.BLOCK_128x128):
            c1, s1 = oracle.quantize_paper(bits, fmt, oracle.COL, group)
            c2, s2 = oracle.quantize_paper(np.ascontiguousarray(bits.T), fmt, oracle.ROW, group)
            assert np.array_equal(c1, c2) and np.array_equal(s1, s2)
    same = np.tile(bits[:1], (128, 1))
    cb, sb = oracle.quantize_paper(same, oracle.FP8, oracle.ROW, oracle.BLOCK_128x128)
    ct, st = oracle.quantize_paper(same, oracle.FP8, oracle.ROW, oracle.TILE_1x128)
    assert np.array_equal(cb, ct) and np.array_equal(np.tile(sb, (128, 1)), st)


def test_stats_paper_is_the_error_of_the_exported_codes():
    rng = np.random.default_rng(124)
    bits = bits_of(rng.standard_t(3, size=(256, 384)))
    x = wl.bf16_bits_to_f32(bits).astype(np.float64)
    for axis in (oracle.ROW, oracle.COL):
        xs = x if axis == oracle.ROW else x.T
        for group in (oracle.TILE_1x128, oracle.BLOCK_128x128):
            if axis == oracle.COL and group == oracle.BLOCK_128x128 and xs.shape[0] % 128:
                continue
            st = oracle.stats_paper(bits, axis, group)
            assert np.isclose(st[0], (x ** 2).sum(), rtol=1e-14)
            for fmt, k in ((oracle.FP4, 1), (oracle.FP8, 2)):
                c, s = oracle.quantize_paper(bits, fmt, axis, group)
                d = oracle.dequantize_paper(c, s, fmt, group) - xs
                assert np.isclose(st[k], (d ** 2).sum(), rtol=1e-13)
    # relative error of a real-valued-scale FP8 cast is bounded by half a unit in the last place (2^-4) of
    # the values that stay normal: a loose but formula-independent sanity bound on the total
    st = oracle.stats_paper(bits, oracle.ROW, oracle.TILE_1x128)
    assert st[2] < (2.0 ** -4) ** 2 * st[0] and st[2] < st[1]


def test_zero_and_non_finite_groups():
    a = np.zeros((2, 256), dtype=np.float32)
    a[1, 5] = np.inf
    a[1, 130] = 3.0
    bits = bits_of(a)
    codes, scales = oracle.quantize_paper(bits, oracle.FP8, oracle.ROW, oracle.TILE_1x128)
    assert scales[0, 0] == 1.0 and scales[0, 1] == 1.0 and not codes[0].any()
    assert np.isnan(scales[1, 0]) and not codes[1, :128].any()
    assert scales[1, 1] == np.float32(448.0) / np.float32(3.0) and codes[1, 130] == 0x7E
    # tiny magnitudes: the scale is capped at 2^126 instead of overflowing
    tiny = np.zeros((1, 128), dtype=np.uint16)
    tiny[0, 0] = 0x0001                                    # smallest bf16 subnormal
    codes, scales = oracle.quantize_paper(tiny, oracle.FP8, oracle.ROW, oracle.TILE_1x128)
    assert scales[0, 0] == np.float32(2.0 ** 126)
