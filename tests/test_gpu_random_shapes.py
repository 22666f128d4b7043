"""GPU parity on seeded random shapes: extents, row strides, formats, scale rules and kernels (the large-tile GEMM
and the general one) drawn at random within the documented limits, every case against the CPU oracle.  The fixed
cases of the other files aim at known boundaries; these look for the ones nobody thought of."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_01410_amd import workloads as wl

from gpu_util import host, host_bf16_as_f64, rel_fro, require_gpu, to_dev

pytestmark = pytest.mark.gpu


def draw_bits(rng, rows, cols):
    """Values over many binades per 32-block, some zeros, some values on rounding ties."""
    a = rng.standard_normal((rows, cols)) * 2.0 ** rng.integers(-12, 12, size=(rows, (cols + 31) // 32)).repeat(32, axis=1)[:, :cols]
    a[rng.random((rows, cols)) < 0.03] = 0.0
    ties = rng.random((rows, cols)) < 0.03
    a[ties] = rng.choice(np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0, 17.0, 19.0, 432.0, 6.0, 448.0]), size=int(ties.sum()))
    return wl.f32_to_bf16_bits(a.astype(np.float32))


def with_stride(bits, pad):
    if not pad:
        return to_dev(bits)
    wide = np.zeros((bits.shape[0], bits.shape[1] + pad), dtype=np.uint16)
    wide[:, :bits.shape[1]] = bits
    return to_dev(wide)[:, :bits.shape[1]]


def check_q(q, bits, fmt, axis, rule):
    want_c, want_s = oracle.quantize(bits, fmt, axis, rule)
    assert np.array_equal(host(q.scales), want_s)
    assert np.array_equal(host(q.codes), want_c)
    g4 = host(q.scales_g4)[:, :want_s.shape[0], :].transpose(1, 0, 2).reshape(want_s.shape[0], -1)
    assert np.array_equal(g4[:, :want_s.shape[1]], want_s)


def check_stats(st, bits, fmt, axis, rule):
    got, want = host(st), oracle.stats(bits, axis, rule)
    k = 2 if fmt == oracle.FP8 else 1
    assert abs(got[0] - want[0]) <= 1e-5 * want[0]
    assert abs(got[k] - want[k]) <= 1e-5 * max(want[k], 1e-300)
    assert np.isnan(got[3 - k])


@pytest.mark.usefixtures("quant_both_unit")
@pytest.mark.parametrize("case", range(24))
def test_quantize_random_shapes(case):
    snip = require_gpu()
    rng = np.random.default_rng(9000 + case)
    rows, cols = 32 * int(rng.integers(1, 13)), 32 * int(rng.integers(1, 25))
    pad = 8 * int(rng.integers(0, 4))
    fr, fc = int(rng.integers(0, 2)), int(rng.integers(0, 2))
    rule = int(rng.integers(0, 2))
    bits = draw_bits(rng, rows, cols)
    x = with_stride(bits, pad)
    print("case", case, rows, cols, pad, fr, fc, rule, flush=True)
    # one call for both orientations, with fused statistics
    sr, sc = snip.alloc_stats(), snip.alloc_stats()
    qr, qc = snip.snip_quantize_both(x, fr, fc, rule, stats_row=sr, stats_col=sc)
    torch.cuda.synchronize()
    check_q(qr, bits, fr, oracle.ROW, rule)
    check_q(qc, bits, fc, oracle.COL, rule)
    check_stats(sr, bits, fr, oracle.ROW, rule)
    check_stats(sc, bits, fc, oracle.COL, rule)
    # the same call with the statistics of both formats
    fr2, fc2 = snip.alloc_stats(), snip.alloc_stats()
    snip.snip_quantize_both(x, fr, fc, rule, out_row=qr, out_col=qc, stats_row=fr2, stats_col=fc2, both_formats=True)
    torch.cuda.synchronize()
    check_q(qr, bits, fr, oracle.ROW, rule)
    check_q(qc, bits, fc, oracle.COL, rule)
    np.testing.assert_allclose(host(fr2), oracle.stats(bits, oracle.ROW, rule), rtol=1e-5)
    np.testing.assert_allclose(host(fc2), oracle.stats(bits, oracle.COL, rule), rtol=1e-5)
    # the single-orientation kernels
    s1, s2 = snip.alloc_stats(), snip.alloc_stats()
    q1 = snip.snip_quantize(x, fc, snip.ROW, rule, stats=s1)
    q2 = snip.snip_quantize(x, fr, snip.COL, rule, stats=s2)
    torch.cuda.synchronize()
    check_q(q1, bits, fc, oracle.ROW, rule)
    check_q(q2, bits, fr, oracle.COL, rule)
    check_stats(s1, bits, fc, oracle.ROW, rule)
    check_stats(s2, bits, fr, oracle.COL, rule)
    # the statistics pass, per line, and its one-read variant
    for axis in (snip.ROW, snip.COL):
        L = rows if axis == snip.ROW else cols
        lines = torch.empty((L, 3), dtype=torch.float32, device="cuda")
        tot = snip.snip_quant_error_stats(x, axis, rule, per_line=lines)
        torch.cuda.synchronize()
        want_tot, want_lines = oracle.stats(bits, axis, rule, per_line=True)
        np.testing.assert_allclose(host(tot), want_tot, rtol=1e-5)
        np.testing.assert_allclose(host(lines), want_lines, rtol=1e-5, atol=1e-30)
    br, bc = snip.snip_quant_error_stats_both(x, rule)
    torch.cuda.synchronize()
    np.testing.assert_allclose(host(br), oracle.stats(bits, oracle.ROW, rule), rtol=1e-5)
    np.testing.assert_allclose(host(bc), oracle.stats(bits, oracle.COL, rule), rtol=1e-5)


@pytest.mark.usefixtures("gemm_tile")
@pytest.mark.parametrize("case", range(16))
def test_gemm_random_shapes(case):
    """Odd cases take extents that admit the large-tile kernel (both output extents above 128, contraction a
    multiple of 256), even ones anything the general kernel takes (contraction a multiple of 32)."""
    snip = require_gpu()
    rng = np.random.default_rng(9500 + case)
    if case % 2:
        I, J, R = int(rng.integers(129, 700)), int(rng.integers(129, 700)), 256 * int(rng.integers(1, 4))
    else:
        I, J, R = int(rng.integers(1, 300)), int(rng.integers(1, 300)), 32 * int(rng.integers(1, 17))
    fa, fb = int(rng.integers(0, 2)), int(rng.integers(0, 2))
    out_dtype = int(rng.integers(0, 2))
    a_bits = wl.f32_to_bf16_bits(rng.standard_normal((I, R)).astype(np.float32))
    b_bits = wl.f32_to_bf16_bits((rng.standard_normal((J, R)) * 0.05).astype(np.float32))
    print("case", case, I, J, R, fa, fb, out_dtype, flush=True)
    aq, bq = snip.snip_quantize(to_dev(a_bits), fa, snip.ROW), snip.snip_quantize(to_dev(b_bits), fb, snip.ROW)
    plan = snip.make_plan((fa, fb, 0, 0, 0, 0))
    ldc = (J + 7) // 8 * 8 + 8 * int(rng.integers(0, 3))          # rows stay 16-byte aligned
    buf = torch.zeros((I, ldc), dtype=torch.float32 if out_dtype else torch.bfloat16, device="cuda")
    y, nrm = snip.snip_gemm_fwd_norm(plan, aq, bq, out=buf[:, :J], out_dtype=out_dtype)
    torch.cuda.synchronize()
    want = oracle.gemm_fwd(oracle.fake_quant(a_bits, fa, oracle.ROW), oracle.fake_quant(b_bits, fb, oracle.ROW))
    got = host(y).astype(np.float64) if out_dtype else host_bf16_as_f64(y)
    assert rel_fro(got, want) <= (1e-4 if out_dtype else 2e-3)
    assert float(host(nrm)[0]) == pytest.approx(float((got ** 2).sum()), rel=5e-6)
    assert float(buf[:, J:].abs().sum()) == 0.0          # nothing written past the row's end
