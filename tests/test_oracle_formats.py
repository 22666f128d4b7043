"""Pins for the oracle's scalar pieces: element grids, round-to-nearest-even cast, block
scale.  Every expected value here comes from a closed form, an enumeration, an exact
rational brute force written independently in Python, or torch's own float8 type -- never
from the oracle itself and never from the GPU path."""
from fractions import Fraction

import numpy as np
import pytest
import torch

import oracle
from oracle import FP4, FP8, FLOOR, NO_OVERFLOW

E2M1_VALUES = [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


def grid(fmt):
    """Non-negative finite grid as exact rationals, from the textbook field formula."""
    eb, mb, bias = (4, 3, 7) if fmt == FP8 else (2, 1, 1)
    out = []
    for E in range(1 << eb):
        for T in range(1 << mb):
            if fmt == FP8 and E == 15 and T == 7:
                continue
            if E == 0:
                v = Fraction(T, 1 << mb) * Fraction(2) ** (1 - bias)
            else:
                v = (1 + Fraction(T, 1 << mb)) * Fraction(2) ** (E - bias)
            out.append(((E << mb) | T, v))
    return out


def brute_nearest(fmt, v: Fraction):
    """Nearest grid value by exhaustive search; ties to the even code; saturating."""
    g = grid(fmt)
    a = abs(v)
    best = min(g, key=lambda cv: (abs(cv[1] - a), cv[0] & 1))
    return best[0]


# ---- grids ---------------------------------------------------------------------------

def test_e2m1_grid_enumeration():
    vals = [oracle.decode(FP4, c) for c in range(8)]
    assert vals == E2M1_VALUES
    assert [oracle.decode(FP4, 8 + c) for c in range(1, 8)] == [-v for v in E2M1_VALUES[1:]]
    assert np.signbit(oracle.decode(FP4, 8)) and oracle.decode(FP4, 8) == 0.0
    assert oracle.fmt_max(FP4) == 6.0


def test_e4m3_grid_enumeration():
    vals = [oracle.decode(FP8, c) for c in range(0x7F)]
    assert len(vals) == 127 and len(set(vals)) == 127
    assert all(b > a for a, b in zip(vals, vals[1:]))           # monotone in the code
    assert vals[0] == 0.0 and vals[1] == 2.0 ** -9 and vals[8] == 2.0 ** -6
    assert vals[-1] == 448.0 == oracle.fmt_max(FP8)
    assert np.isnan(oracle.decode(FP8, 0x7F)) and np.isnan(oracle.decode(FP8, 0xFF))
    for c, v in grid(FP8):
        assert oracle.decode(FP8, c) == float(v)
        assert oracle.decode(FP8, 0x80 | c) == -float(v)


def test_e4m3_decode_matches_torch_float8():
    codes = torch.arange(256, dtype=torch.uint8)
    ref = codes.view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = np.array([oracle.decode(FP8, c) for c in range(256)])
    assert np.array_equal(np.isnan(ref), np.isnan(got))
    ok = ~np.isnan(ref)
    assert np.array_equal(ref[ok], got[ok])
    assert np.array_equal(np.signbit(ref[ok]), np.signbit(got[ok]))


# ---- cast ----------------------------------------------------------------------------

@pytest.mark.parametrize("fmt", [FP4, FP8])
def test_encode_grid_values_are_fixed_points(fmt):
    for c, v in grid(fmt):
        assert oracle.encode_rne(fmt, float(v)) == c
        sign = 0x80 if fmt == FP8 else 0x8
        assert oracle.encode_rne(fmt, -float(v)) == (sign | c)
    assert oracle.encode_rne(fmt, -0.0) == (0x80 if fmt == FP8 else 0x8)


def test_e2m1_tie_table():
    table = {0.25: 0.0, 0.75: 1.0, 1.25: 1.0, 1.75: 2.0, 2.5: 2.0, 3.5: 4.0, 5.0: 4.0}
    for v, want in table.items():
        assert oracle.decode(FP4, oracle.encode_rne(FP4, v)) == want
        assert oracle.decode(FP4, oracle.encode_rne(FP4, -v)) == -want


def test_e4m3_tie_table():
    table = {2.0 ** -10: 0.0, 3 * 2.0 ** -10: 2.0 ** -8, 17.0: 16.0, 19.0: 20.0, 432.0: 448.0,
             2.0 ** -6 - 2.0 ** -10: 2.0 ** -6}
    for v, want in table.items():
        assert oracle.decode(FP8, oracle.encode_rne(FP8, v)) == want


@pytest.mark.parametrize("fmt", [FP4, FP8])
def test_encode_matches_exact_brute_force(fmt):
    g = [v for _, v in grid(fmt)]
    pts = set(g)
    for a, b in zip(g, g[1:]):
        mid = (a + b) / 2
        eps = (b - a) / 1024
        pts.update([mid, mid - eps, mid + eps, a + eps, b - eps])
    top = g[-1]
    pts.update([top + Fraction(1, 7), top * 2, top * 1000, Fraction(1, 1 << 20)])
    rng = np.random.default_rng(5)
    pts.update(Fraction(float(x)) for x in np.abs(rng.standard_normal(300)) * float(top) / 3)
    for v in pts:
        want = brute_nearest(fmt, v)
        assert oracle.encode_rne(fmt, float(v)) == want, (fmt, float(v))
        sign = 0x80 if fmt == FP8 else 0x8
        assert oracle.encode_rne(fmt, -float(v)) == (sign | want)


def test_e4m3_encode_matches_torch_in_range():
    rng = np.random.default_rng(11)
    v = np.concatenate([rng.standard_normal(4000) * 100, rng.standard_normal(2000) * 0.01,
                        np.array([447.9, 448.0, 463.9, -463.9, 1e-4, 0.0])])
    v = v[np.abs(v) < 464].astype(np.float32)          # torch overflows to NaN beyond that
    ref = torch.from_numpy(v).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    got = np.array([oracle.encode_rne(FP8, float(x)) for x in v], dtype=np.uint8)
    assert np.array_equal(ref, got)


def test_encode_saturates():
    assert oracle.encode_rne(FP8, 1e9) == 0x7E and oracle.encode_rne(FP8, -465.0) == 0xFE
    assert oracle.encode_rne(FP4, 6.01) == 0x7 and oracle.encode_rne(FP4, -100.0) == 0xF


# ---- block scale ---------------------------------------------------------------------

def all_positive_bf16():
    bits = np.arange(1, 0x7F80, dtype=np.uint32)            # subnormals .. largest finite
    return bits, (bits << 16).view(np.float32).astype(np.float64)


@pytest.mark.parametrize("fmt,emax,top", [(FP8, 8, 448), (FP4, 2, 6)])
def test_scale_closed_forms_every_bf16_amax(fmt, emax, top):
    bits, vals = all_positive_bf16()
    step = 37                                              # every 37th value plus the edges
    pick = np.unique(np.concatenate([np.arange(0, len(vals), step), [0, 1, 127, 128, len(vals) - 1]]))
    for i in pick:
        amax = Fraction(float(vals[i]))
        n = amax.numerator.bit_length() - amax.denominator.bit_length()
        if Fraction(2) ** n > amax:
            n -= 1                                         # floor(log2 amax), exactly
        b_floor = oracle.scale_byte(fmt, FLOOR, float(amax))
        b_safe = oracle.scale_byte(fmt, NO_OVERFLOW, float(amax))
        assert b_floor == min(max(n - emax, -127), 127) + 127
        # smallest power of two that keeps amax / 2^e inside the format
        e = -127
        while amax / Fraction(2) ** e > top:
            e += 1
        assert b_safe == e + 127
        if e > -127:
            assert Fraction(top, 2) < amax / Fraction(2) ** e <= top
        # the two rules differ exactly when the mantissa of amax exceeds the format's
        m = amax / Fraction(2) ** n
        mmax = Fraction(top) / Fraction(2) ** emax
        if n - emax >= -127:
            assert (b_safe != b_floor) == (m > mmax)
        assert 0 <= b_safe <= 254 and 0 <= b_floor <= 254


def test_scale_special_blocks():
    for fmt in (FP4, FP8):
        for rule in (NO_OVERFLOW, FLOOR):
            assert oracle.scale_byte(fmt, rule, 0.0) == 0
            assert oracle.scale_byte(fmt, rule, float("inf")) == 0xFF
            assert oracle.scale_byte(fmt, rule, float("nan")) == 0xFF
    assert oracle.scale_byte(FP8, NO_OVERFLOW, 448.0) == 127
    assert oracle.scale_byte(FP8, NO_OVERFLOW, 450.0) == 128
    assert oracle.scale_byte(FP8, FLOOR, 480.0) == 127
    assert oracle.scale_byte(FP4, NO_OVERFLOW, 6.0) == 127
    assert oracle.scale_byte(FP4, NO_OVERFLOW, 6.5) == 128
    assert oracle.scale_byte(FP4, FLOOR, 7.5) == 127
    assert oracle.scale_byte(FP4, NO_OVERFLOW, 1.0) == 127 - 2


def _golden(name):
    import os
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", name)
    return [l.split() for l in open(path) if l.strip() and not l.startswith("#")]


def test_element_values_from_the_mx_specification():
    """Decode (and encode back) against the value table kept under tests/golden/."""
    import math
    for fmt_name, code, value in _golden("mx_element_values.txt"):
        fmt = oracle.FP4 if fmt_name == "fp4" else oracle.FP8
        got = oracle.decode(fmt, int(code, 16))
        if value == "nan":
            assert math.isnan(got)
            continue
        want = float(value)
        assert got == want and math.copysign(1.0, got) == math.copysign(1.0, want), (fmt_name, code)
        assert oracle.encode_rne(fmt, want) == int(code, 16)
