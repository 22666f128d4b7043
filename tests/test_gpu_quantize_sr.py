"""GPU parity: FP4 quantization with stochastic rounding against the CPU oracle, bit for bit (both sides
implement the same byte stream and the same threshold rule, each in its own code), plus the statistical
property the method wants from it."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_01410_amd import workloads as wl

from gpu_util import host, require_gpu, to_dev
from test_gpu_quantize import wide_range_bits

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("quant_col_unit")]


@pytest.mark.parametrize("axis", [oracle.ROW, oracle.COL])
@pytest.mark.parametrize("rule", [oracle.NO_OVERFLOW, oracle.FLOOR])
@pytest.mark.parametrize("seed", [0, 0x9E3779B97F4A7C15])
def test_sr_ragged_wide_range(axis, rule, seed):
    snip = require_gpu()
    rng = np.random.default_rng(90 + axis)
    rows, cols = (203, 1632) if axis == oracle.ROW else (416, 1344)      # several units, ragged tails
    bits = wide_range_bits(rng, rows, cols)
    q = snip.snip_quantize_sr_fp4(to_dev(bits), axis, rule, seed)
    torch.cuda.synchronize()
    want_c, want_s = oracle.quantize_sr_fp4(bits, axis, rule, seed)
    assert np.array_equal(host(q.scales), want_s)
    assert np.array_equal(host(q.codes), want_c)
    # scales (and the grouped copy) are those of the nearest-even path
    q_ne = snip.snip_quantize(to_dev(bits), snip.FP4, axis, rule)
    torch.cuda.synchronize()
    assert torch.equal(q.scales, q_ne.scales)
    sr = want_s.shape[0]
    assert torch.equal(q.scales_g4[:-1, :sr], q_ne.scales_g4[:-1, :sr])


def test_sr_gradient_shaped_tensor_with_row_pitch():
    """Config-1 gradient (the tensor the method rounds stochastically), source with a padded row pitch."""
    snip = require_gpu()
    lay = wl.make_layer(wl.CONFIGS[1])
    bits = lay.dY["lin"]
    wide = np.zeros((bits.shape[0], bits.shape[1] + 64), dtype=np.uint16)
    wide[:, :bits.shape[1]] = bits
    x = to_dev(wide)[:, :bits.shape[1]]
    for axis in (oracle.ROW, oracle.COL):
        q = snip.snip_quantize_sr_fp4(x, axis, oracle.NO_OVERFLOW, seed=1234)
        torch.cuda.synchronize()
        want_c, want_s = oracle.quantize_sr_fp4(bits, axis, oracle.NO_OVERFLOW, 1234)
        assert np.array_equal(host(q.codes), want_c) and np.array_equal(host(q.scales), want_s)


def test_sr_every_bf16_magnitude_up_to_the_block_maximum():
    """One block per row: element 0 is 6 * 2^k (fixes the scale), the others sweep bf16 magnitudes from far
    below the grid to the maximum, so every branch of the rounding (zero neighbourhood, the three spacings,
    grid points, the top value) meets many random bytes."""
    snip = require_gpu()
    mags = np.arange(0x3000, 0x40C1, dtype=np.uint16)            # 2^-31 .. 6.0
    n = (len(mags) + 30) // 31
    bits = np.zeros((n, 32), dtype=np.uint16)
    bits[:, 0] = 0x40C0                                           # 6.0
    flat = np.zeros(n * 31, dtype=np.uint16)
    flat[:len(mags)] = mags
    flat[1::2] |= 0x8000                                          # alternate signs
    bits[:, 1:] = flat.reshape(n, 31)
    rows = ((n + 31) // 32) * 32                                  # so that the column variant's blocked extent fits
    full = np.zeros((rows, 32), dtype=np.uint16)
    full[:n] = bits
    for seed in (3, 4, 5):
        q = snip.snip_quantize_sr_fp4(to_dev(full), oracle.ROW, oracle.NO_OVERFLOW, seed)
        torch.cuda.synchronize()
        want_c, want_s = oracle.quantize_sr_fp4(full, oracle.ROW, oracle.NO_OVERFLOW, seed)
        assert np.array_equal(host(q.codes), want_c) and np.array_equal(host(q.scales), want_s)


def test_sr_is_unbiased_where_nearest_even_is_not():
    """Mean of the dequantized tensor over 256 seeds: within sampling error of x; nearest-even stays off."""
    snip = require_gpu()
    rng = np.random.default_rng(91)
    bits = wl.f32_to_bf16_bits(rng.standard_normal((32, 256)).astype(np.float32))
    x = wl.bf16_bits_to_f32(bits).astype(np.float64)
    xd = to_dev(bits)
    acc = np.zeros_like(x)
    n = 256
    for seed in range(n):
        q = snip.snip_quantize_sr_fp4(xd, oracle.ROW, oracle.NO_OVERFLOW, seed)
        torch.cuda.synchronize()
        acc += oracle.dequantize(host(q.codes), host(q.scales), oracle.FP4)
    mean = acc / n
    scale = 2.0 ** (host(q.scales).astype(np.float64) - 127.0).repeat(32, axis=1)
    assert np.all(np.abs(mean - x) <= scale * (5.0 / np.sqrt(n) + 1.0 / 256))
    c, s = oracle.quantize(bits, oracle.FP4, oracle.ROW)
    assert np.abs(oracle.dequantize(c, s, oracle.FP4) - x).mean() > 3 * np.abs(mean - x).mean()


def test_sr_codes_feed_the_gemm():
    """A stochastically rounded gradient is an ordinary FP4 operand: dgrad on it matches the oracle's product
    of the oracle's stochastically rounded tensor."""
    snip = require_gpu()
    rng = np.random.default_rng(92)
    M, N, K = 288, 320, 256
    dY = wl.f32_to_bf16_bits((1e-3 * rng.standard_normal((M, N))).astype(np.float32))
    W = wl.f32_to_bf16_bits((0.02 * rng.standard_normal((N, K))).astype(np.float32))
    plan = snip.make_plan((1,) * 6)
    dyq = snip.snip_quantize_sr_fp4(to_dev(dY), snip.ROW, seed=77)
    wq = snip.snip_quantize(to_dev(W), snip.FP4, snip.COL)
    dx = snip.snip_gemm_dgrad(plan, dyq, wq, out_dtype=snip.OUT_FP32)
    torch.cuda.synchronize()
    c, s = oracle.quantize_sr_fp4(dY, oracle.ROW, oracle.NO_OVERFLOW, 77)
    want = oracle.gemm_dgrad(oracle.dequantize(c, s, oracle.FP4), oracle.fake_quant(W, oracle.FP4, oracle.COL))
    got = host(dx).astype(np.float64)
    assert np.linalg.norm(got - want) <= 1e-4 * np.linalg.norm(want)


def test_sr_rejects_fp8_output_and_empty_is_fine():
    snip = require_gpu()
    x = torch.zeros((32, 64), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(snip.SnipError):
        snip.snip_quantize_sr_fp4(x, out=snip.alloc_qtensor(32, 64, snip.FP8))
    e = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    q = snip.snip_quantize_sr_fp4(e)
    torch.cuda.synchronize()
    assert q.rows == 0
