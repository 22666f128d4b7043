"""Pins for the oracle's tensor-level functions: whole-tensor quantize / dequantize, the
three products, the statistics.  Expected values come from an independent exact-rational
brute force, from hand-computed blocks, from invariants the definitions imply, and from
numpy's own matmul -- never from the oracle itself and never from the GPU path."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import COL, FLOOR, FP4, FP8, NO_OVERFLOW, ROW
from paper_2602_01410_amd.workloads import bf16_bits_to_f32, f32_to_bf16_bits

from test_oracle_formats import brute_nearest, grid


def bits(a):
    return f32_to_bf16_bits(np.asarray(a, dtype=np.float32))


def unpack_codes(codes, fmt):
    if fmt == FP8:
        return codes
    out = np.empty((codes.shape[0], codes.shape[1] * 2), dtype=np.uint8)
    out[:, 0::2] = codes & 0xF
    out[:, 1::2] = codes >> 4
    return out


def brute_quantize_rows(x_f64, fmt, rule):
    """Exact-rational reference for row tiles, written without reference to the C code."""
    top = Fraction(448 if fmt == FP8 else 6)
    emax = 8 if fmt == FP8 else 2
    R, C = x_f64.shape
    codes = np.zeros((R, C), dtype=np.uint8)
    scales = np.zeros((R, C // 32), dtype=np.uint8)
    sign_bit = 0x80 if fmt == FP8 else 0x8
    for r in range(R):
        for b in range(C // 32):
            blk = [Fraction(float(v)) for v in x_f64[r, b * 32:(b + 1) * 32]]
            amax = max(abs(v) for v in blk)
            e = -127
            if amax > 0:
                if rule == NO_OVERFLOW:
                    while amax / Fraction(2) ** e > top and e < 127:
                        e += 1
                else:
                    while Fraction(2) ** (e + emax + 1) <= amax and e < 127:
                        e += 1
            scales[r, b] = e + 127
            for i, v in enumerate(blk):
                c = brute_nearest(fmt, min(abs(v) / Fraction(2) ** e, top))
                neg = np.signbit(x_f64[r, b * 32 + i])
                codes[r, b * 32 + i] = c | (sign_bit if neg else 0)
    return codes, scales


@pytest.mark.parametrize("fmt", [FP4, FP8])
@pytest.mark.parametrize("rule", [NO_OVERFLOW, FLOOR])
def test_quantize_matches_exact_brute_force(fmt, rule):
    rng = np.random.default_rng(100 + fmt * 2 + rule)
    x = rng.standard_normal((3, 96)).astype(np.float32)
    x[1, :32] *= 1e-3
    x[2, 32:64] *= 300.0
    x[0, 5] = 0.0
    x[0, 6] = -0.0
    xb = bits(x)
    codes, scales = oracle.quantize(xb, fmt, ROW, rule)
    want_c, want_s = brute_quantize_rows(bf16_bits_to_f32(xb).astype(np.float64), fmt, rule)
    assert np.array_equal(scales, want_s)
    assert np.array_equal(unpack_codes(codes, fmt), want_c)


def test_hand_computed_fp4_block():
    # amax 6 pins e = 0; the rest walks the E2M1 tie table and the sign of zero
    blk = [6.0, 0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, -0.25, -2.5, 0.0, -0.0, 0.1, 5.9, -6.0, 2.0]
    x = np.zeros((1, 32), dtype=np.float32)
    x[0, :16] = blk
    codes, scales = oracle.quantize(bits(x), FP4, ROW, NO_OVERFLOW)
    assert scales[0, 0] == 127
    got = unpack_codes(codes, FP4)[0, :16].tolist()
    #        6   .25 .75 1.25 1.75 2.5 3.5 5  -.25 -2.5  0  -0   .1  5.9  -6   2
    assert got == [7, 0, 2, 2, 4, 4, 6, 6, 8, 12, 0, 8, 0, 7, 15, 4]
    # low nibble holds the even element
    assert codes[0, 0] == (0 << 4 | 7) and codes[0, 1] == (2 << 4 | 2)


def test_hand_computed_fp8_block():
    blk = [448.0, 432.0, 17.0, 19.0, 2.0 ** -10, 3 * 2.0 ** -10, -17.0, 0.0]
    x = np.zeros((1, 32), dtype=np.float32)
    x[0, :8] = blk
    codes, scales = oracle.quantize(bits(x), FP8, ROW, NO_OVERFLOW)
    assert scales[0, 0] == 127
    # 448 = 0x7E; 432 ties to 448; 17 -> 16 (E=11,T=0 -> 0x58); 19 -> 20 (0x5A);
    # 2^-10 -> 0; 3*2^-10 -> 2^-8 (T=2); -17 -> -16
    assert codes[0, :8].tolist() == [0x7E, 0x7E, 0x58, 0x5A, 0x00, 0x02, 0xD8, 0x00]


@pytest.mark.parametrize("fmt,top_codes", [(FP4, [6, 7]), (FP8, list(range(0x78, 0x7F)))])
@pytest.mark.parametrize("rule", [NO_OVERFLOW, FLOOR])
def test_round_trip_of_representable_blocks(fmt, top_codes, rule):
    """A block of grid values times 2^e whose largest element sits in the top binade comes
    back with the same codes and the same e."""
    rng = np.random.default_rng(7)
    ncodes = 0x7F if fmt == FP8 else 8
    for e in (-20, -3, 0, 5, 30):
        c = rng.integers(0, ncodes, size=(4, 64)).astype(np.uint8)
        c[:, 0] = rng.choice(top_codes, size=4)
        c[:, 32] = rng.choice(top_codes, size=4)
        sgn = rng.integers(0, 2, size=c.shape).astype(np.uint8) * (0x80 if fmt == FP8 else 0x8)
        full = c | sgn
        vals = np.array([[oracle.decode(fmt, int(v)) for v in row] for row in full]) * 2.0 ** e
        xb = bits(vals)
        assert np.array_equal(bf16_bits_to_f32(xb).astype(np.float64), vals)   # exact in bf16
        codes, scales = oracle.quantize(xb, fmt, ROW, rule)
        assert np.all(scales == e + 127)
        assert np.array_equal(unpack_codes(codes, fmt), full)


@pytest.mark.parametrize("fmt", [FP4, FP8])
def test_error_is_zero_on_representable_tensors(fmt):
    rng = np.random.default_rng(8)
    ncodes = 0x7F if fmt == FP8 else 8
    # bf16 keeps 8 significant bits: every E2M1/E4M3 value times 2^e is exact
    c = rng.integers(0, ncodes, size=(8, 128))
    vals = np.array([[oracle.decode(fmt, int(v)) for v in row] for row in c])
    vals *= np.where(rng.random(vals.shape) < 0.5, -1.0, 1.0) * 2.0 ** rng.integers(-9, 9, size=(8, 1))
    xb = bits(vals)
    q = oracle.fake_quant(xb, fmt, ROW, NO_OVERFLOW)
    assert np.array_equal(q, vals)
    s = oracle.stats(xb, ROW, NO_OVERFLOW)
    assert s[0] == np.sum(vals ** 2)
    assert s[2 if fmt == FP8 else 1] == 0.0
    if fmt == FP4:
        assert s[2] == 0.0          # E2M1 values are E4M3 values too


def test_floor_rule_saturates_where_no_overflow_does_not():
    x = np.zeros((1, 32), dtype=np.float32)
    x[0, 0] = 240.0       # mantissa 1.875 > 1.75: floor scales it to 480 > 448
    x[0, 1] = 1.0
    xb = bits(x)
    assert oracle.fake_quant(xb, FP8, ROW, NO_OVERFLOW)[0, 0] == 240.0
    assert oracle.fake_quant(xb, FP8, ROW, FLOOR)[0, 0] == 224.0      # 448 * 2^-1
    assert oracle.quantize(xb, FP8, ROW, FLOOR)[1][0, 0] == 127 - 1
    assert oracle.quantize(xb, FP8, ROW, NO_OVERFLOW)[1][0, 0] == 127


@pytest.mark.parametrize("fmt", [FP4, FP8])
@pytest.mark.parametrize("rule", [NO_OVERFLOW, FLOOR])
def test_power_of_two_scaling_invariance(fmt, rule):
    rng = np.random.default_rng(9)
    x = rng.standard_normal((4, 64)).astype(np.float32)
    xb = bits(x)
    base_c, base_s = oracle.quantize(xb, fmt, ROW, rule)
    for k in (-7, 3, 11):
        xk = bits(bf16_bits_to_f32(xb) * np.float32(2.0 ** k))
        c, s = oracle.quantize(xk, fmt, ROW, rule)
        assert np.array_equal(c, base_c)
        assert np.array_equal(s.astype(int), base_s.astype(int) + k)


@pytest.mark.parametrize("fmt", [FP4, FP8])
def test_column_tiles_equal_row_tiles_of_the_transpose(fmt):
    rng = np.random.default_rng(10)
    x = rng.standard_normal((64, 40)) * 4.0 ** rng.integers(-6, 6, size=(64, 40))
    xb = bits(x.astype(np.float32))
    c1, s1 = oracle.quantize(xb, fmt, COL)
    c2, s2 = oracle.quantize(np.ascontiguousarray(xb.T), fmt, ROW)
    assert c1.shape == c2.shape and np.array_equal(c1, c2) and np.array_equal(s1, s2)
    q_col = oracle.fake_quant(xb, fmt, COL)
    q_row_t = oracle.fake_quant(np.ascontiguousarray(xb.T), fmt, ROW)
    assert q_col.shape == (64, 40) and np.array_equal(q_col, q_row_t.T)
    # and the two tilings really differ
    assert not np.array_equal(q_col[:32, :32], oracle.fake_quant(np.ascontiguousarray(xb[:32, :32]), fmt, ROW))


@pytest.mark.parametrize("fmt,bound", [(FP4, 1.0 / 3.0), (FP8, 1.0 / 14.0)])
def test_error_bound_and_scale_range(fmt, bound):
    rng = np.random.default_rng(12)
    x = (rng.standard_t(3, size=(16, 256)) * 10.0 ** rng.integers(-6, 3, size=(16, 1))).astype(np.float32)
    xb = bits(x)
    xv = bf16_bits_to_f32(xb).astype(np.float64)
    codes, scales = oracle.quantize(xb, fmt, ROW, NO_OVERFLOW)
    q = oracle.dequantize(codes, scales, fmt)
    amax = np.abs(xv).reshape(16, 8, 32).max(axis=2)
    top = 448.0 if fmt == FP8 else 6.0
    ratio = amax / 2.0 ** (scales.astype(np.float64) - 127)
    assert np.all(ratio <= top) and np.all(ratio > top / 2)
    err = np.abs(q - xv).reshape(16, 8, 32)
    assert np.all(err < bound * amax[:, :, None] + 1e-300)
    rel = np.linalg.norm(q - xv) / np.linalg.norm(xv)
    assert rel < (0.2 if fmt == FP4 else 0.05)


def test_special_blocks():
    x = np.zeros((2, 64), dtype=np.float32)
    x[0, 3] = -0.0
    x[1, 40] = np.inf
    x[1, 0] = 1.0
    xb = bits(x)
    xb[1, 41] = 0x7FC0            # a NaN in the same block as the infinity
    for fmt in (FP4, FP8):
        codes, scales = oracle.quantize(xb, fmt, ROW)
        u = unpack_codes(codes, fmt)
        assert scales[0].tolist() == [0, 0]                       # all-zero blocks: 2^-127
        assert u[0, 3] == (0x80 if fmt == FP8 else 0x8) and u[0].sum() == u[0, 3]
        assert scales[1].tolist()[1] == 0xFF and np.all(u[1, 32:] == 0)
        assert scales[1, 0] == oracle.scale_byte(fmt, NO_OVERFLOW, 1.0)
        assert np.all(np.isnan(oracle.dequantize(codes, scales, fmt)[1, 32:]))
    # bf16 subnormal block: scale clamps at 2^-127, values still fit
    t = np.zeros((1, 32), dtype=np.uint16)
    t[0, 0] = 0x0001
    t[0, 1] = 0x0078            # 120 * 2^-133 -> 1.875 * 2^-127 after scaling
    c, s = oracle.quantize(t, FP8, ROW)
    assert s[0, 0] == 0
    assert oracle.dequantize(c, s, FP8)[0, 1] == oracle.bf16_to_f64(0x0078)


def test_bad_arguments_are_rejected():
    x = np.zeros((4, 48), dtype=np.uint16)
    with pytest.raises(ValueError):
        oracle.quantize(x, FP8, ROW)            # 48 is not a multiple of 32
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((48, 32), dtype=np.uint16), FP8, COL)
    with pytest.raises(ValueError):
        oracle.quantize(np.zeros((32, 32), dtype=np.uint16), 2, ROW)


# ---- the three products ---------------------------------------------------------------

def test_products_equal_numpy_on_integers_exactly():
    rng = np.random.default_rng(13)
    M, N, K = 9, 7, 11
    X = rng.integers(-6, 7, size=(M, K)).astype(np.float64)
    W = rng.integers(-6, 7, size=(N, K)).astype(np.float64)
    dY = rng.integers(-6, 7, size=(M, N)).astype(np.float64)
    assert np.array_equal(oracle.gemm_fwd(X, W), X @ W.T)
    assert np.array_equal(oracle.gemm_dgrad(dY, W), dY @ W)
    assert np.array_equal(oracle.gemm_wgrad(dY, X), dY.T @ X)


def test_products_equal_numpy_on_reals_and_are_not_interchangeable():
    rng = np.random.default_rng(14)
    M, N, K = 33, 20, 45
    X, W, dY = rng.standard_normal((M, K)), rng.standard_normal((N, K)), rng.standard_normal((M, N))
    np.testing.assert_allclose(oracle.gemm_fwd(X, W), X @ W.T, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.gemm_dgrad(dY, W), dY @ W, rtol=0, atol=1e-12)
    np.testing.assert_allclose(oracle.gemm_wgrad(dY, X), dY.T @ X, rtol=0, atol=1e-12)
    # one-hot operands read back rows / columns of the other operand
    E = np.eye(K)
    assert np.array_equal(oracle.gemm_fwd(X, E), X)
    assert np.array_equal(oracle.gemm_dgrad(np.eye(N), W), W)
    assert np.array_equal(oracle.gemm_wgrad(np.eye(M)[:, :5], X), X[:5])
    # dgrad(dY, W) is fwd(dY, W^T)
    np.testing.assert_allclose(oracle.gemm_dgrad(dY, W), oracle.gemm_fwd(dY, W.T.copy()), atol=1e-12)


# ---- statistics -----------------------------------------------------------------------

def test_stats_hand_computed_block():
    x = np.zeros((1, 32), dtype=np.float32)
    x[0, 0], x[0, 1], x[0, 2] = 6.0, 0.25, 2.5
    s = oracle.stats(bits(x), ROW)
    # FP4: e = 0, 0.25 -> 0 (err .25), 2.5 -> 2 (err .5).  FP8: amax 6 -> e = -6, all exact.
    assert s.tolist() == [36.0 + 0.0625 + 6.25, 0.0625 + 0.25, 0.0]


@pytest.mark.parametrize("axis", [ROW, COL])
@pytest.mark.parametrize("rule", [NO_OVERFLOW, FLOOR])
def test_stats_equal_error_of_exported_codes(axis, rule):
    rng = np.random.default_rng(15)
    x = rng.standard_t(3, size=(64, 96)).astype(np.float32)
    xb = bits(x)
    xv = bf16_bits_to_f32(xb).astype(np.float64)
    s, lines = oracle.stats(xb, axis, rule, per_line=True)
    src = xv if axis == ROW else xv.T
    want = [np.sum(src ** 2)]
    want_lines = [np.sum(src ** 2, axis=1)]
    for fmt in (FP4, FP8):
        c, sc = oracle.quantize(xb, fmt, axis, rule)
        d = oracle.dequantize(c, sc, fmt) - src
        want.append(np.sum(d ** 2))
        want_lines.append(np.sum(d ** 2, axis=1))
    np.testing.assert_allclose(s, want, rtol=1e-13)
    np.testing.assert_allclose(lines, np.stack(want_lines, axis=1), rtol=1e-13)
    np.testing.assert_allclose(lines.sum(axis=0), s, rtol=1e-13)
    assert s[1] > s[2] > 0                  # FP4 is coarser than FP8
