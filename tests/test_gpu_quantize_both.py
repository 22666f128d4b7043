"""GPU parity: snip_quantize_both (row-block and column-block quantization from one read) against the CPU
oracle, bit for bit, for every pair of formats; fused statistics within 1e-5."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_01410_amd import workloads as wl

from gpu_util import host, require_gpu, to_dev
from test_gpu_quantize import wide_range_bits

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("quant_both_unit")]

FMTS = [oracle.FP8, oracle.FP4]
RULES = [oracle.NO_OVERFLOW, oracle.FLOOR]
TOL = 1e-5


def check_g4(q, want_s):
    g4 = host(q.scales_g4)
    sr, nkb = want_s.shape
    pad = np.zeros((sr, g4.shape[0] * 4), dtype=np.uint8)
    pad[:, :nkb] = want_s
    want_g4 = pad.reshape(sr, g4.shape[0], 4).transpose(1, 0, 2)
    got_g4 = g4[:, :sr, :].copy()
    if nkb % 4:                       # bytes of blocks past the end are unspecified
        got_g4[-1, :, nkb % 4:] = 0
    assert np.array_equal(got_g4, want_g4)


def check(snip, bits, fmt_r, fmt_c, rule, ld_pad=0, with_stats=False):
    if ld_pad:
        wide = np.zeros((bits.shape[0], bits.shape[1] + ld_pad), dtype=np.uint16)
        wide[:, :bits.shape[1]] = bits
        x = to_dev(wide)[:, :bits.shape[1]]
    else:
        x = to_dev(bits)
    sr, sc = (snip.alloc_stats(), snip.alloc_stats()) if with_stats else (None, None)
    qr, qc = snip.snip_quantize_both(x, fmt_r, fmt_c, rule, stats_row=sr, stats_col=sc)
    torch.cuda.synchronize()
    for q, fmt, axis in ((qr, fmt_r, oracle.ROW), (qc, fmt_c, oracle.COL)):
        want_c, want_s = oracle.quantize(bits, fmt, axis, rule)
        assert np.array_equal(host(q.scales), want_s), (fmt, axis)
        assert np.array_equal(host(q.codes), want_c), (fmt, axis)
        check_g4(q, want_s)
    if with_stats:
        for st, fmt, axis in ((sr, fmt_r, oracle.ROW), (sc, fmt_c, oracle.COL)):
            got, want = host(st), oracle.stats(bits, axis, rule)
            k = 2 if fmt == oracle.FP8 else 1
            assert abs(got[0] - want[0]) <= TOL * want[0]
            assert abs(got[k] - want[k]) <= TOL * want[k]
            assert np.isnan(got[3 - k])


@pytest.mark.parametrize("fmt_r", FMTS)
@pytest.mark.parametrize("fmt_c", FMTS)
@pytest.mark.parametrize("rule", RULES)
def test_wide_range_ragged(fmt_r, fmt_c, rule):
    """Nine row blocks (one full FP4 unit of eight plus one; two FP8 units plus one) and 9.25 column groups:
    ragged in both directions, scale rows that are not a whole number of dwords."""
    snip = require_gpu()
    rng = np.random.default_rng(100 + fmt_r + 2 * fmt_c + 4 * rule)
    bits = np.ascontiguousarray(wide_range_bits(rng, 288, 1216)[:, :1184])
    check(snip, bits, fmt_r, fmt_c, rule)


@pytest.mark.parametrize("fmt_r", FMTS)
@pytest.mark.parametrize("fmt_c", FMTS)
def test_whole_groups_strided_rows_and_stats(fmt_r, fmt_c):
    """Extents that are multiples of 128 (dword scale stores on both sides), rows with a stride, fused statistics."""
    snip = require_gpu()
    rng = np.random.default_rng(7 + fmt_r + 2 * fmt_c)
    bits = wl.f32_to_bf16_bits((rng.standard_t(3, size=(384, 1024)) * 0.3).astype(np.float32))
    check(snip, bits, fmt_r, fmt_c, oracle.NO_OVERFLOW, ld_pad=40, with_stats=True)


@pytest.mark.parametrize("fmt", FMTS)
def test_nonfinite_and_zero_blocks(fmt):
    snip = require_gpu()
    rng = np.random.default_rng(5)
    bits = wl.f32_to_bf16_bits(rng.standard_normal((64, 160)).astype(np.float32))
    bits[3, 40] = 0x7F80       # +inf
    bits[10, 100] = 0xFF80     # -inf
    bits[20, 5] = 0x7FC0       # NaN
    bits[33:40, :] = 0
    bits[35, 7] = 0x8000       # -0 inside an all-zero block
    check(snip, bits, fmt, fmt, oracle.NO_OVERFLOW)


def test_config1_tensors():
    snip = require_gpu()
    lay = wl.make_layer(wl.CONFIGS[1])
    for bits in (lay.X["x"], lay.W["lin"], lay.dY["lin"]):
        check(snip, bits, oracle.FP4, oracle.FP8, oracle.NO_OVERFLOW, with_stats=True)
        check(snip, bits, oracle.FP8, oracle.FP4, oracle.NO_OVERFLOW, with_stats=True)


@pytest.mark.parametrize("fmt_r", FMTS)
@pytest.mark.parametrize("fmt_c", FMTS)
@pytest.mark.parametrize("rule", RULES)
def test_statistics_of_both_formats_from_the_same_pass(fmt_r, fmt_c, rule):
    """both_formats=True: the complete triple for either direction (what the statistics pass delivers), next to the
    same codes and scales."""
    snip = require_gpu()
    rng = np.random.default_rng(300 + fmt_r + 2 * fmt_c + 4 * rule)
    bits = wl.f32_to_bf16_bits((rng.standard_t(3, size=(288, 1184)) * 0.3).astype(np.float32))
    sr, sc = snip.alloc_stats(), snip.alloc_stats()
    qr, qc = snip.snip_quantize_both(to_dev(bits), fmt_r, fmt_c, rule, stats_row=sr, stats_col=sc, both_formats=True)
    torch.cuda.synchronize()
    for q, st, fmt, axis in ((qr, sr, fmt_r, oracle.ROW), (qc, sc, fmt_c, oracle.COL)):
        want_c, want_s = oracle.quantize(bits, fmt, axis, rule)
        assert np.array_equal(host(q.scales), want_s) and np.array_equal(host(q.codes), want_c)
        np.testing.assert_allclose(host(st), oracle.stats(bits, axis, rule), rtol=TOL)


def test_equals_single_orientation_calls_and_is_deterministic():
    """Same bytes as the two separate calls (which the other tests tie to the oracle) on a tensor too large for
    the oracle to be run in the test: 2048 x 4224."""
    snip = require_gpu()
    rng = np.random.default_rng(11)
    x = to_dev(wl.f32_to_bf16_bits(rng.standard_normal((2048, 4224)).astype(np.float32)))
    for fmt_r, fmt_c in ((snip.FP4, snip.FP4), (snip.FP8, snip.FP4), (snip.FP4, snip.FP8), (snip.FP8, snip.FP8)):
        s = [snip.alloc_stats() for _ in range(6)]
        qr, qc = snip.snip_quantize_both(x, fmt_r, fmt_c, stats_row=s[0], stats_col=s[1])
        qr2, qc2 = snip.snip_quantize_both(x, fmt_r, fmt_c, stats_row=s[2], stats_col=s[3])
        a = snip.snip_quantize(x, fmt_r, snip.ROW, stats=s[4])
        b = snip.snip_quantize(x, fmt_c, snip.COL, stats=s[5])
        torch.cuda.synchronize()
        for got, want in ((qr, a), (qc, b), (qr2, a), (qc2, b)):
            assert torch.equal(got.codes, want.codes) and torch.equal(got.scales, want.scales)
            same_g4 = torch.equal(got.scales_g4[:, :got.rows], want.scales_g4[:, :want.rows])     # rows past the end: padding
            assert same_g4
        assert host(s[0]).tobytes() == host(s[2]).tobytes() and host(s[1]).tobytes() == host(s[3]).tobytes()
        for got, want in ((s[0], s[4]), (s[1], s[5])):
            g, w = host(got), host(want)
            ok = ~np.isnan(w)
            assert np.array_equal(np.isnan(g), np.isnan(w))
            assert np.all(np.abs(g[ok] - w[ok]) <= TOL * w[ok])


def test_empty_and_argument_errors():
    snip = require_gpu()
    x = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    s0, s1 = snip.alloc_stats(), snip.alloc_stats()
    qr, qc = snip.snip_quantize_both(x, snip.FP8, snip.FP4, stats_row=s0, stats_col=s1)
    torch.cuda.synchronize()
    assert qr.codes.numel() == 0 and qc.codes.numel() == 0
    assert host(s0)[0] == 0.0 and host(s1)[0] == 0.0
    y = torch.zeros((48, 64), dtype=torch.bfloat16, device="cuda")          # rows not a multiple of 32
    with pytest.raises(snip.SnipError):
        snip.snip_quantize_both(y, snip.FP8, snip.FP8)
    z = torch.zeros((64, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(snip.SnipError):
        snip.snip_quantize_both(z, snip.FP8, snip.FP8, stats_row=s0)       # only one statistics output


@pytest.mark.parametrize("shape", [(2080, 1056), (4096, 4096), (32, 160)])
def test_wave_and_workgroup_units_write_the_same_bytes(shape, monkeypatch):
    """The two work distributions and the launcher's own pick agree on every output byte; the statistics agree to
    the tolerance (their partial sums are combined in another order)."""
    snip = require_gpu()
    rng = np.random.default_rng(5)
    x = to_dev(wl.f32_to_bf16_bits((rng.standard_normal(shape) * np.exp(rng.normal(0, 3, (shape[0], 1)))).astype(np.float32)))
    for fmt_r, fmt_c in ((snip.FP4, snip.FP8), (snip.FP8, snip.FP4)):
        outs = {}
        for unit in ("wave", "workgroup", None):
            if unit is None:
                monkeypatch.delenv("SNIP_QUANT_BOTH_UNIT", raising=False)
            else:
                monkeypatch.setenv("SNIP_QUANT_BOTH_UNIT", unit)
            sr, sc = snip.alloc_stats(), snip.alloc_stats()
            qr, qc = snip.snip_quantize_both(x, fmt_r, fmt_c, stats_row=sr, stats_col=sc, both_formats=True)
            torch.cuda.synchronize()
            outs[unit] = (qr, qc, host(sr), host(sc))
        for unit in ("workgroup", None):
            for i in (0, 1):
                got, want = outs[unit][i], outs["wave"][i]
                assert torch.equal(got.codes, want.codes) and torch.equal(got.scales, want.scales)
                assert torch.equal(got.scales_g4[:, :got.rows], want.scales_g4[:, :want.rows])
            for i in (2, 3):
                np.testing.assert_allclose(outs[unit][i], outs["wave"][i], rtol=TOL)
