"""GPU parity of the GEMMs and of the statistics totals at benchmark size, sharper than a Frobenius norm over
a sample: every linear of the 7B-shaped configuration under the plan the benchmark times (quantized the way
the benchmark quantizes, bf16 and fp32 output, per-row bounds), exact-integer operands at every contraction
extent (hence every pipeline stage count) the benchmark runs, on grids that give some workgroups a second
tile, and the statistics totals of one full tensor per configuration directly against the oracle."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_01410_amd import workloads as wl

from gpu_util import host, host_bf16_as_f64, require_gpu, to_dev

pytestmark = pytest.mark.gpu
TOL_BF16, TOL_F32 = 2e-3, 1e-4


def sample(n, k, rng):
    return np.unique(np.concatenate([[0, n - 1], rng.integers(0, n, size=k)]))


def check_rows(got_bf16, got_f32, want, what):
    """Sampled output rows: relative Frobenius error over the sample and per row, both output types."""
    for got, tol in ((host_bf16_as_f64(got_bf16), TOL_BF16), (host(got_f32).astype(np.float64), TOL_F32)):
        assert got.shape == want.shape, what
        assert np.linalg.norm(got - want) <= tol * np.linalg.norm(want), what
        nw = np.linalg.norm(want, axis=1)
        row_err = np.linalg.norm(got - want, axis=1) / np.where(nw > 0, nw, 1.0)
        assert row_err.max() <= 2 * tol, (what, float(row_err.max()))


@pytest.mark.parametrize("linear", ["q", "k", "v", "o", "gate", "up", "down"])
def test_config4_mix50_every_linear(linear):
    snip = require_gpu()
    cfg = wl.CONFIGS[4]
    li = next(i for i, l in enumerate(cfg.linears) if l.name == linear)
    lin = cfg.linears[li]
    entry = wl.make_plan(cfg, "mix50")[li]
    fx, fw, gdy, gw, wdy, wx = entry
    rng = np.random.default_rng(700 + li)
    X, W, dY = wl.make_tensor(cfg, "X", lin.x_group), wl.make_tensor(cfg, "W", lin.name), wl.make_tensor(cfg, "dY", lin.name)
    M, N, K = cfg.M, lin.N, lin.K
    plan = snip.make_plan(entry)
    # quantized as the benchmark step does it: both orientations of a tensor from one call, statistics fused
    st = [snip.alloc_stats() for _ in range(6)]
    xq_r, xq_c = snip.snip_quantize_both(to_dev(X), fx, wx, stats_row=st[0], stats_col=st[1], both_formats=True)
    wq_r, wq_c = snip.snip_quantize_both(to_dev(W), fw, gw, stats_row=st[2], stats_col=st[3], both_formats=True)
    dyq_r, dyq_c = snip.snip_quantize_both(to_dev(dY), gdy, wdy, stats_row=st[4], stats_col=st[5], both_formats=True)
    outs = {}
    for dt in (snip.OUT_BF16, snip.OUT_FP32):
        outs[dt] = (snip.snip_gemm_fwd(plan, xq_r, wq_r, out_dtype=dt), snip.snip_gemm_dgrad(plan, dyq_r, wq_c, out_dtype=dt),
                    snip.snip_gemm_wgrad(plan, dyq_c, xq_c, out_dtype=dt))
    torch.cuda.synchronize()
    ms, ns = sample(M, 10, rng), sample(N, 10, rng)
    Wh = oracle.fake_quant(W, fw, oracle.ROW)
    want = oracle.gemm_fwd(oracle.fake_quant(X[ms], fx, oracle.ROW), Wh)
    check_rows(outs[0][0][ms], outs[1][0][ms], want, "fwd")
    Wh = oracle.fake_quant(W, gw, oracle.COL)
    want = oracle.gemm_dgrad(oracle.fake_quant(dY[ms], gdy, oracle.ROW), Wh)
    check_rows(outs[0][1][ms], outs[1][1][ms], want, "dgrad")
    del Wh
    Xh = oracle.fake_quant(X, wx, oracle.COL)
    want = oracle.gemm_wgrad(oracle.fake_quant(np.ascontiguousarray(dY[:, ns]), wdy, oracle.COL), Xh)
    check_rows(outs[0][2][ns], outs[1][2][ns], want, "wgrad")
    del Xh
    # the fused statistics of the weight (the smallest of the three tensors): the complete record against the oracle
    np.testing.assert_allclose(host(st[2]), oracle.stats(W, oracle.ROW), rtol=1e-5)
    np.testing.assert_allclose(host(st[3]), oracle.stats(W, oracle.COL), rtol=1e-5)


@pytest.mark.parametrize("fmt", [0, 1])
@pytest.mark.parametrize("R", [4096, 11008, 16384])
@pytest.mark.parametrize("I,J", [(2816, 6400), (2600, 6504)])
def test_exact_integers_at_benchmark_contractions(fmt, R, I, J):
    """Operands on the FP4 grid with magnitudes up to 1 (rows of A scaled by 1 or 2): every product is a multiple of
    1/4 and every partial sum stays below 2^17 quarter units, so any summation order is exact in fp32 and the output
    must equal the oracle's element for element.  11 x 25 (or 11 x 26 ragged) tiles of 256 x 256: more tiles than
    compute units, so some workgroups walk into a second tile; 16/43/64 (FP4) and 32/86/128 (FP8) stages per tile."""
    snip = require_gpu()
    rng = np.random.default_rng(800 + R // 64 + fmt)
    vals = np.array([-1.0, -0.5, 0.0, 0.5, 1.0])
    A = rng.choice(vals, size=(I, R)) * 2.0 ** rng.integers(0, 2, size=(I, 1))
    B = rng.choice(vals, size=(J, R))
    A, B = wl.f32_to_bf16_bits(A.astype(np.float32)), wl.f32_to_bf16_bits(B.astype(np.float32))
    aq, bq = snip.snip_quantize(to_dev(A), fmt, snip.ROW), snip.snip_quantize(to_dev(B), fmt, snip.ROW)
    y = snip.snip_gemm_fwd((fmt,) * 6, aq, bq, out_dtype=snip.OUT_FP32)
    yb = snip.snip_gemm_fwd((fmt,) * 6, aq, bq, out_dtype=snip.OUT_BF16)
    torch.cuda.synchronize()
    ms = sample(I, 24, rng)
    want = oracle.gemm_fwd(oracle.fake_quant(A[ms], fmt, oracle.ROW), oracle.fake_quant(B, fmt, oracle.ROW))
    assert np.array_equal(host(y[ms]).astype(np.float64), want)
    # bf16 output: the same exact sums rounded once to nearest even
    want_b = host_bf16_as_f64(torch.from_numpy(want.astype(np.float32)).to(torch.bfloat16))
    assert np.array_equal(host_bf16_as_f64(yb[ms]), want_b)
    # every tile took part: column sums of the whole output against the oracle's from row sums of A (exact as well)
    col_sum = host(y.double().sum(dim=0))
    a_sum = oracle.fake_quant(A, fmt, oracle.ROW).sum(axis=0, keepdims=True)               # [1, R]
    want_cs = oracle.gemm_fwd(a_sum, oracle.fake_quant(B, fmt, oracle.ROW))[0]
    assert np.array_equal(col_sum, want_cs)


@pytest.mark.parametrize("config", [2, 3, 4, 5])
def test_statistics_totals_of_a_full_tensor_against_the_oracle(config):
    """The output gradient of the configuration's largest linear, in full: totals of the stand-alone statistics call
    (both directions from one read) and of the statistics fused into the two-orientation quantize call, each directly
    against the oracle's fp64 sums over the whole tensor."""
    snip = require_gpu()
    cfg = wl.CONFIGS[config]
    lin = max(cfg.linears, key=lambda l: l.N * l.K)
    T = wl.make_tensor(cfg, "dY", lin.name)
    want_r, want_c = oracle.stats(T, oracle.ROW), oracle.stats(T, oracle.COL)
    t = to_dev(T)
    both_r, both_c = snip.snip_quant_error_stats_both(t)
    st_r, st_c = snip.alloc_stats(), snip.alloc_stats()
    snip.snip_quantize_both(t, snip.FP4, snip.FP8, stats_row=st_r, stats_col=st_c, both_formats=True)
    one_r, one_c = snip.snip_quant_error_stats(t, snip.ROW), snip.snip_quant_error_stats(t, snip.COL)
    torch.cuda.synchronize()
    for got, want in ((both_r, want_r), (both_c, want_c), (st_r, want_r), (st_c, want_c), (one_r, want_r), (one_c, want_c)):
        np.testing.assert_allclose(host(got), want, rtol=1e-5)
