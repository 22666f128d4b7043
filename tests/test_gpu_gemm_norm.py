"""GPU parity: the GEMM variants that also return the squared Frobenius norm of their stored output
(Sec. 3.1 Step 1: norms of Y, dX, dW), and the loss-divergence estimate built from them (Sec. 4.2).

Tolerance of the norm: 1e-4 relative.  The stored output differs from the oracle's exact product by the
fp32 accumulation (<= 3e-5 relative Frobenius, zero mean) and, for bf16, by rounding decisions that flip
where the two sides sit on opposite sides of a rounding boundary; both perturb the SUM of squares by far
less than they perturb single elements.  The kernel adds 64 or 128 squares per lane and 64 lanes per wave
in fp32 (<= 2e-6 relative), then waves in double.  Measured differences are 1e-7 .. 1e-5."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_01410_amd import workloads as wl

from gpu_util import host, host_bf16_as_f64, require_gpu, to_dev

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("gemm_tile")]
TOL_NORM = 1e-4


def gpu_layer(snip, X, W, dY, entry, out_dtype):
    fx, fw, gdy, gw, wdy, wx = entry
    dX_, dW_, ddY = to_dev(X), to_dev(W), to_dev(dY)
    plan = snip.make_plan(entry)
    y, ny = snip.snip_gemm_fwd_norm(plan, snip.snip_quantize(dX_, fx, snip.ROW), snip.snip_quantize(dW_, fw, snip.ROW),
                                    out_dtype=out_dtype)
    dx, ndx = snip.snip_gemm_dgrad_norm(plan, snip.snip_quantize(ddY, gdy, snip.ROW), snip.snip_quantize(dW_, gw, snip.COL),
                                        out_dtype=out_dtype)
    dw, ndw = snip.snip_gemm_wgrad_norm(plan, snip.snip_quantize(ddY, wdy, snip.COL), snip.snip_quantize(dX_, wx, snip.COL),
                                        out_dtype=out_dtype)
    torch.cuda.synchronize()
    return (y, dx, dw), [float(host(t)[0]) for t in (ny, ndx, ndw)]


def oracle_layer(X, W, dY, entry):
    fx, fw, gdy, gw, wdy, wx = entry
    y = oracle.gemm_fwd(oracle.fake_quant(X, fx, oracle.ROW), oracle.fake_quant(W, fw, oracle.ROW))
    dx = oracle.gemm_dgrad(oracle.fake_quant(dY, gdy, oracle.ROW), oracle.fake_quant(W, gw, oracle.COL))
    dw = oracle.gemm_wgrad(oracle.fake_quant(dY, wdy, oracle.COL), oracle.fake_quant(X, wx, oracle.COL))
    return y, dx, dw


def as_f64(t):
    return host_bf16_as_f64(t) if t.dtype == torch.bfloat16 else host(t).astype(np.float64)


@pytest.mark.parametrize("out_dtype", [0, 1])
@pytest.mark.parametrize("entry", [(0,) * 6, (1,) * 6, (0, 1, 1, 0, 0, 1)])
def test_norms_small_general_kernel(entry, out_dtype):
    """Ragged shapes below the large-tile kernel's threshold and with a contraction extent it does not take."""
    snip = require_gpu()
    rng = np.random.default_rng(70)
    M, N, K = 160, 96, 224
    X = wl.f32_to_bf16_bits(rng.standard_normal((M, K)).astype(np.float32))
    W = wl.f32_to_bf16_bits((0.02 * rng.standard_normal((N, K))).astype(np.float32))
    dY = wl.f32_to_bf16_bits((1e-3 * rng.standard_normal((M, N))).astype(np.float32))
    outs, norms = gpu_layer(snip, X, W, dY, entry, out_dtype)
    for c, got, out in zip(oracle_layer(X, W, dY, entry), norms, outs):
        assert got == pytest.approx(oracle.output_sum_sq(c, out_dtype), rel=TOL_NORM)
        # and it is the norm of what was stored, to summation rounding
        assert got == pytest.approx(float((as_f64(out) ** 2).sum()), rel=5e-6)


@pytest.mark.parametrize("out_dtype", [0, 1])
@pytest.mark.parametrize("entry", [(1,) * 6, (0,) * 6, (1, 0, 0, 1, 1, 0)])
def test_norms_large_tile_kernel_ragged(entry, out_dtype):
    """Several 256 x 256 tiles with ragged edges in both output dimensions: rows and columns past the
    end of the matrix must not count."""
    snip = require_gpu()
    rng = np.random.default_rng(71)
    M, N, K = 544, 416, 512
    X = wl.f32_to_bf16_bits(rng.standard_t(3, size=(M, K)).astype(np.float32))
    W = wl.f32_to_bf16_bits((0.02 * rng.standard_normal((N, K))).astype(np.float32))
    dY = wl.f32_to_bf16_bits((1e-4 * rng.standard_normal((M, N))).astype(np.float32))
    outs, norms = gpu_layer(snip, X, W, dY, entry, out_dtype)
    for c, got, out in zip(oracle_layer(X, W, dY, entry), norms, outs):
        assert got == pytest.approx(oracle.output_sum_sq(c, out_dtype), rel=TOL_NORM)
        assert got == pytest.approx(float((as_f64(out) ** 2).sum()), rel=5e-6)


def test_norm_exact_on_integers_and_deterministic():
    """Operands in {-1, 0, 1}: outputs are integers of magnitude <= ~40, a lane's 128 squares and a wave's
    64 lane sums stay below 2^24, so every fp32 partial is exact and the norm must equal the oracle's to
    the last bit; two runs must agree bit for bit."""
    snip = require_gpu()
    rng = np.random.default_rng(72)
    M, N, K = 320, 288, 256
    vals = np.array([-1, 0, 0, 1.0])
    X = wl.f32_to_bf16_bits(rng.choice(vals, size=(M, K)).astype(np.float32))
    W = wl.f32_to_bf16_bits(rng.choice(vals, size=(N, K)).astype(np.float32))
    dY = wl.f32_to_bf16_bits(rng.choice(vals, size=(M, N)).astype(np.float32))
    entry = (1,) * 6
    _, a = gpu_layer(snip, X, W, dY, entry, snip.OUT_FP32)
    _, b = gpu_layer(snip, X, W, dY, entry, snip.OUT_FP32)
    assert a == b
    want = [oracle.output_sum_sq(c, oracle.OUT_FP32) for c in oracle_layer(X, W, dY, entry)]
    assert a == want


def test_norm_of_empty_output_is_zero():
    snip = require_gpu()
    plan = snip.make_plan((0,) * 6)
    a = snip.alloc_qtensor(0, 64, snip.FP8)
    b = snip.alloc_qtensor(32, 64, snip.FP8)
    b.codes.zero_(); b.scales.zero_()
    out = torch.empty((0, 32), dtype=torch.bfloat16, device="cuda")
    ws = torch.empty(64, dtype=torch.uint8, device="cuda")
    _, n = snip.snip_gemm_fwd_norm(plan, a, b, out=out, workspace=ws)
    torch.cuda.synchronize()
    assert float(host(n)[0]) == 0.0


def test_loss_divergence_of_config1_layer():
    """End to end for one linear: norms of dX and dW from the GEMM epilogues, quantization-error norms of
    X and W from the statistics pass, combined by the host function, against the same chain in the oracle."""
    snip = require_gpu()
    cfg = wl.CONFIGS[1]
    lay = wl.make_layer(cfg)
    lin = cfg.linears[0]
    X, W, dY = lay.X[lin.x_group], lay.W[lin.name], lay.dY[lin.name]
    for fmt, field in ((snip.FP8, 2), (snip.FP4, 1)):
        entry = (fmt,) * 6
        _, (ny, ndx, ndw) = gpu_layer(snip, X, W, dY, entry, snip.OUT_BF16)
        sx = host(snip.snip_quant_error_stats(to_dev(X), snip.ROW))
        sw = host(snip.snip_quant_error_stats(to_dev(W), snip.ROW))
        torch.cuda.synchronize()
        got = snip.snip_loss_divergence(ndx, sx[field], cfg.M, ndw, sw[field], lin.N, lin.K)
        _, odx, odw = oracle_layer(X, W, dY, entry)
        want = oracle.loss_divergence(oracle.output_sum_sq(odx), oracle.stats(X, oracle.ROW)[field], cfg.M,
                                      oracle.output_sum_sq(odw), oracle.stats(W, oracle.ROW)[field], lin.N, lin.K)
        assert got == pytest.approx(want, rel=TOL_NORM)
        assert got > 0.0
