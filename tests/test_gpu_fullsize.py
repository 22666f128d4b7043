"""GPU parity at the full sizes of the Llama-shaped configurations, in the launch configuration the
benchmark times (bf16 output, grouped scales, 256x256-tile kernel).  The oracle cannot afford the
whole fp64 product at these sizes, so outputs are checked on sampled rows that it computes one by one
(each sampled output row uses the complete contraction), quantized codes and scales bit for bit on
sampled slabs, and the statistics on sampled lines plus the identity total = sum of lines."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_01410_amd import workloads as wl

from gpu_util import host, host_bf16_as_f64, require_gpu, to_dev

pytestmark = pytest.mark.gpu
TOL = 2e-3


def sample(n, k, rng):
    idx = np.unique(np.concatenate([[0, n - 1], rng.integers(0, n, size=k)]))
    return idx


@pytest.mark.parametrize("config,plan_name,linear", [
    (2, "fp4", "q"), (2, "fp4", "down"), (3, "mix60", "q"), (3, "mix60", "k"), (4, "mix50", "q"), (4, "fp8", "q"),
    (4, "fp4", "down"), (4, "tensor", "gate"), (5, "mix50", "q"), (5, "mix50", "k")])
def test_linear_at_full_size(config, plan_name, linear):
    snip = require_gpu()
    cfg = wl.CONFIGS[config]
    li = next(i for i, l in enumerate(cfg.linears) if l.name == linear)
    lin = cfg.linears[li]
    entry = wl.make_plan(cfg, plan_name)[li]
    fx, fw, gdy, gw, wdy, wx = entry
    rng = np.random.default_rng(500 + config)
    X = wl.make_tensor(cfg, "X", lin.x_group)
    W = wl.make_tensor(cfg, "W", lin.name)
    dY = wl.make_tensor(cfg, "dY", lin.name)
    M, N, K = cfg.M, lin.N, lin.K
    dX_, dW_, ddY = to_dev(X), to_dev(W), to_dev(dY)
    plan = snip.make_plan(entry)

    xq_r = snip.snip_quantize(dX_, fx, snip.ROW)
    wq_r = snip.snip_quantize(dW_, fw, snip.ROW)
    dyq_r = snip.snip_quantize(ddY, gdy, snip.ROW)
    wq_c = snip.snip_quantize(dW_, gw, snip.COL)
    dyq_c = snip.snip_quantize(ddY, wdy, snip.COL)
    xq_c = snip.snip_quantize(dX_, wx, snip.COL)
    y = snip.snip_gemm_fwd(plan, xq_r, wq_r)
    dx = snip.snip_gemm_dgrad(plan, dyq_r, wq_c)
    dw = snip.snip_gemm_wgrad(plan, dyq_c, xq_c)
    torch.cuda.synchronize()

    ms = sample(M, 12, rng)          # token rows
    ns = sample(N, 12, rng)          # output features
    ks = sample(K, 12, rng)          # input features

    # ---- quantize: bit-exact on sampled slabs (row slabs for ROW, column slabs for COL) ----
    c, s = oracle.quantize(X[ms], fx, oracle.ROW)
    assert np.array_equal(host(xq_r.codes[ms]), c) and np.array_equal(host(xq_r.scales[ms]), s)
    c, s = oracle.quantize(np.ascontiguousarray(X[:, ks]), wx, oracle.COL)
    assert np.array_equal(host(xq_c.codes[ks]), c) and np.array_equal(host(xq_c.scales[ks]), s)
    c, s = oracle.quantize(np.ascontiguousarray(dY[:, ns]), wdy, oracle.COL)
    assert np.array_equal(host(dyq_c.codes[ns]), c) and np.array_equal(host(dyq_c.scales[ns]), s)
    c, s = oracle.quantize(W[ns], fw, oracle.ROW)
    assert np.array_equal(host(wq_r.codes[ns]), c) and np.array_equal(host(wq_r.scales[ns]), s)

    # ---- GEMMs: sampled output rows, each over the full contraction ----
    Wh_row = oracle.fake_quant(W, fw, oracle.ROW)
    want = oracle.gemm_fwd(oracle.fake_quant(X[ms], fx, oracle.ROW), Wh_row)
    got = host_bf16_as_f64(y[ms])
    assert np.linalg.norm(got - want) <= TOL * np.linalg.norm(want)
    del Wh_row
    Wh_col = oracle.fake_quant(W, gw, oracle.COL)
    want = oracle.gemm_dgrad(oracle.fake_quant(dY[ms], gdy, oracle.ROW), Wh_col)
    got = host_bf16_as_f64(dx[ms])
    assert np.linalg.norm(got - want) <= TOL * np.linalg.norm(want)
    del Wh_col
    Xh_col = oracle.fake_quant(X, wx, oracle.COL)
    dYh_cols = oracle.fake_quant(np.ascontiguousarray(dY[:, ns]), wdy, oracle.COL)      # [M, len(ns)]
    want = oracle.gemm_wgrad(dYh_cols, Xh_col)                                           # [len(ns), K]
    got = host_bf16_as_f64(dw[ns])
    assert np.linalg.norm(got - want) <= TOL * np.linalg.norm(want)
    del Xh_col

    # ---- norm-returning variants: same stored output bit for bit; the norm is that of the stored output,
    #      and on the sampled rows the stored squares agree with the oracle's rounded product ----
    dx2, ndx = snip.snip_gemm_dgrad_norm(plan, dyq_r, wq_c)
    dw2, ndw = snip.snip_gemm_wgrad_norm(plan, dyq_c, xq_c)
    torch.cuda.synchronize()
    assert torch.equal(dx2, dx) and torch.equal(dw2, dw)
    for out, n in ((dx, ndx), (dw, ndw)):
        stored = float((out.double() ** 2).sum())
        assert float(host(n)[0]) == pytest.approx(stored, rel=5e-6)
    assert float((dw[ns].double() ** 2).sum()) == pytest.approx(oracle.output_sum_sq(want), rel=1e-4)

    # ---- both orientations from one call, with fused statistics (what the benchmark step calls): the same bytes
    #      as the single-orientation calls sampled against the oracle above; statistics against the statistics pass ----
    for t_dev, f_r, f_c, want_r, want_c in ((dX_, fx, wx, xq_r, xq_c), (ddY, gdy, wdy, dyq_r, dyq_c), (dW_, fw, gw, wq_r, wq_c)):
        st_r, st_c = snip.alloc_stats(), snip.alloc_stats()
        got_r, got_c = snip.snip_quantize_both(t_dev, f_r, f_c, stats_row=st_r, stats_col=st_c)
        ref_r, ref_c = snip.snip_quant_error_stats(t_dev, snip.ROW), snip.snip_quant_error_stats(t_dev, snip.COL)
        torch.cuda.synchronize()
        for got, want, st, ref, f in ((got_r, want_r, st_r, ref_r, f_r), (got_c, want_c, st_c, ref_c, f_c)):
            assert torch.equal(got.codes, want.codes) and torch.equal(got.scales, want.scales)
            same_g4 = torch.equal(got.scales_g4[:, :got.rows], want.scales_g4[:, :want.rows])
            assert same_g4
            k = 2 if f == snip.FP8 else 1
            np.testing.assert_allclose(host(st)[[0, k]], host(ref)[[0, k]], rtol=1e-5)
            assert np.isnan(host(st)[3 - k])
        # the same call with the statistics of both formats: the complete record of the statistics pass
        got_r, got_c = snip.snip_quantize_both(t_dev, f_r, f_c, out_row=got_r, out_col=got_c, stats_row=st_r, stats_col=st_c,
                                               both_formats=True)
        torch.cuda.synchronize()
        assert torch.equal(got_r.codes, want_r.codes) and torch.equal(got_c.codes, want_c.codes)
        np.testing.assert_allclose(host(st_r), host(ref_r), rtol=1e-5)
        np.testing.assert_allclose(host(st_c), host(ref_c), rtol=1e-5)
        del got_r, got_c

    # ---- the one-read statistics of both block directions (what the benchmark step calls) agree with the
    #      per-direction totals checked below ----
    both_r, both_c = snip.snip_quant_error_stats_both(ddY)
    torch.cuda.synchronize()
    np.testing.assert_allclose(host(both_r), host(snip.snip_quant_error_stats(ddY, snip.ROW)), rtol=1e-5)
    np.testing.assert_allclose(host(both_c), host(snip.snip_quant_error_stats(ddY, snip.COL)), rtol=1e-5)

    # ---- statistics: sampled lines against the oracle, and total = sum of lines ----
    for t_dev, t_host, axis, idx in ((ddY, dY, snip.ROW, ms), (dX_, X, snip.COL, ks)):
        L = t_host.shape[0] if axis == snip.ROW else t_host.shape[1]
        lines = torch.empty((L, 3), dtype=torch.float32, device="cuda")
        tot = snip.snip_quant_error_stats(t_dev, axis, per_line=lines)
        torch.cuda.synchronize()
        slab = t_host[idx] if axis == snip.ROW else np.ascontiguousarray(t_host[:, idx])
        _, want_lines = oracle.stats(slab, axis, per_line=True)
        np.testing.assert_allclose(host(lines)[idx], want_lines, rtol=1e-5)
        np.testing.assert_allclose(host(tot), host(lines).astype(np.float64).sum(axis=0), rtol=1e-5)
