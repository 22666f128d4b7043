"""GPU parity: the three GEMMs against the oracle's fp64 product of the dequantized operands."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_01410_amd import workloads as wl

from gpu_util import host, host_bf16_as_f64, rel_fro, require_gpu, to_dev

pytestmark = [pytest.mark.gpu, pytest.mark.usefixtures("gemm_tile")]
TOL_BF16 = 2e-3      # relative Frobenius error, bf16 output (one RNE to bf16 costs ~1.7e-3)
TOL_F32 = 1e-4       # fp32 output: the matrix core sums the 64 products of one instruction with a
                     # shared alignment, not as IEEE fp32 adds; measured 1e-5 .. 3e-5


def layer_gemms(snip, X, W, dY, entry, out_dtype):
    """Run quantize + the three GEMMs of one linear on the GPU."""
    fx, fw, gdy, gw, wdy, wx = entry
    dX_, dW_ = to_dev(X), to_dev(W)
    ddY = to_dev(dY)
    plan = snip.make_plan(entry)
    y = snip.snip_gemm_fwd(plan, snip.snip_quantize(dX_, fx, snip.ROW), snip.snip_quantize(dW_, fw, snip.ROW),
                           out_dtype=out_dtype)
    dx = snip.snip_gemm_dgrad(plan, snip.snip_quantize(ddY, gdy, snip.ROW), snip.snip_quantize(dW_, gw, snip.COL),
                              out_dtype=out_dtype)
    dw = snip.snip_gemm_wgrad(plan, snip.snip_quantize(ddY, wdy, snip.COL), snip.snip_quantize(dX_, wx, snip.COL),
                              out_dtype=out_dtype)
    torch.cuda.synchronize()
    return y, dx, dw


def oracle_gemms(X, W, dY, entry):
    fx, fw, gdy, gw, wdy, wx = entry
    y = oracle.gemm_fwd(oracle.fake_quant(X, fx, oracle.ROW), oracle.fake_quant(W, fw, oracle.ROW))
    dx = oracle.gemm_dgrad(oracle.fake_quant(dY, gdy, oracle.ROW), oracle.fake_quant(W, gw, oracle.COL))
    dw = oracle.gemm_wgrad(oracle.fake_quant(dY, wdy, oracle.COL), oracle.fake_quant(X, wx, oracle.COL))
    return y, dx, dw


def as_f64(t):
    return host_bf16_as_f64(t) if t.dtype == torch.bfloat16 else host(t).astype(np.float64)


@pytest.mark.parametrize("entry", [(0,) * 6, (1,) * 6, (0, 1, 1, 0, 0, 1), (1, 0, 0, 1, 1, 0)])
def test_small_integers_are_exact(entry):
    """Operands whose quantization is exact and whose products and partial sums need fewer than
    21 bits (element range 2^3.6, row scales 2^-1..2^1, at most 384 terms): every summation order
    is exact in fp32, so the output must equal the oracle exactly.  This pins every operand and
    scale register layout."""
    snip = require_gpu()
    rng = np.random.default_rng(40)
    M, N, K = 160, 224, 384
    vals = np.array([-6, -4, -3, -2, -1.5, -1, -.5, 0, .5, 1, 1.5, 2, 3, 4, 6.0])
    def draw(r, c, scale_rows):
        a = rng.choice(vals, size=(r, c))
        a *= 2.0 ** rng.integers(-1, 2, size=(r, 1)) if scale_rows else 1.0
        return wl.f32_to_bf16_bits(a.astype(np.float32))
    X, W, dY = draw(M, K, True), draw(N, K, True), draw(M, N, True)
    got = layer_gemms(snip, X, W, dY, entry, snip.OUT_FP32)
    want = oracle_gemms(X, W, dY, entry)
    for g, w in zip(got, want):
        assert np.array_equal(host(g).astype(np.float64), w)


@pytest.mark.parametrize("out_dtype,tol", [(0, TOL_BF16), (1, TOL_F32)])
def test_config1_full(out_dtype, tol):
    snip = require_gpu()
    cfg = wl.CONFIGS[1]
    lay = wl.make_layer(cfg)
    entry = wl.make_plan(cfg, "fp8")[0]
    got = layer_gemms(snip, lay.X["x"], lay.W["lin"], lay.dY["lin"], entry, out_dtype)
    want = oracle_gemms(lay.X["x"], lay.W["lin"], lay.dY["lin"], entry)
    for g, w in zip(got, want):
        assert g.shape == w.shape
        assert rel_fro(as_f64(g), w) <= tol


@pytest.mark.parametrize("entry", [(1,) * 6, (0,) * 6, (0, 1, 1, 0, 1, 0)])
@pytest.mark.parametrize("out_dtype,tol", [(0, TOL_BF16), (1, TOL_F32)])
def test_ragged_shapes_all_formats(entry, out_dtype, tol):
    """Tiles with ragged edges in every dimension; contraction extents that are odd multiples
    of 32 (scale rows not dword aligned, last stage partial)."""
    snip = require_gpu()
    rng = np.random.default_rng(41)
    M, N, K = 352, 416, 608          # all multiples of 32 (each is a contraction extent of one GEMM)
    X = wl.f32_to_bf16_bits(rng.standard_t(3, size=(M, K)).astype(np.float32))
    W = wl.f32_to_bf16_bits((rng.standard_normal((N, K)) * 0.02).astype(np.float32))
    dY = wl.f32_to_bf16_bits((rng.standard_normal((M, N)) * 1e-3).astype(np.float32))
    got = layer_gemms(snip, X, W, dY, entry, out_dtype)
    want = oracle_gemms(X, W, dY, entry)
    for g, w in zip(got, want):
        assert rel_fro(as_f64(g), w) <= tol


@pytest.mark.parametrize("fx,fw", [(0, 0), (1, 1), (0, 1), (1, 0)])
@pytest.mark.parametrize("out_dtype,tol", [(0, TOL_BF16), (1, TOL_F32)])
def test_large_tile_kernel_ragged_rows(fx, fw, out_dtype, tol):
    """Contraction extent a multiple of 128 and more than one 128-tile in each direction: the
    256x256-tile kernel runs; 300 and 520 rows leave ragged tiles in both directions."""
    snip = require_gpu()
    rng = np.random.default_rng(43 + fx + 2 * fw)
    M, N, K = 300, 520, 640
    X = wl.f32_to_bf16_bits((rng.standard_t(3, size=(M, K)) * 2.0 ** rng.integers(-6, 6, size=(M, 1))).astype(np.float32))
    W = wl.f32_to_bf16_bits((rng.standard_normal((N, K)) * 0.02).astype(np.float32))
    y = snip.snip_gemm_fwd((fx, fw, 0, 0, 0, 0), snip.snip_quantize(to_dev(X), fx, snip.ROW),
                           snip.snip_quantize(to_dev(W), fw, snip.ROW), out_dtype=out_dtype)
    torch.cuda.synchronize()
    want = oracle.gemm_fwd(oracle.fake_quant(X, fx, oracle.ROW), oracle.fake_quant(W, fw, oracle.ROW))
    assert y.shape == want.shape
    assert rel_fro(as_f64(y), want) <= tol
    # per-row check: a wrong scale row or a swapped tile would hide in a global norm
    g = as_f64(y)
    row_err = np.linalg.norm(g - want, axis=1) / np.linalg.norm(want, axis=1)
    assert row_err.max() <= 4 * tol


@pytest.mark.parametrize("entry", [(0,) * 6, (1,) * 6, (0, 1, 1, 0, 0, 1)])
def test_large_tile_kernel_exact_integers(entry):
    """Exactness test again at a size served by the 256x256-tile kernel (several stages of its ring)."""
    snip = require_gpu()
    rng = np.random.default_rng(44)
    M, N, K = 384, 640, 1152
    vals = np.array([-6, -4, -3, -2, -1.5, -1, -.5, 0, .5, 1, 1.5, 2, 3, 4, 6.0])
    def draw(r, c):
        a = rng.choice(vals, size=(r, c)) * 2.0 ** rng.integers(-1, 2, size=(r, 1))
        return wl.f32_to_bf16_bits(a.astype(np.float32))
    X, W, dY = draw(M, K), draw(N, K), draw(M, N)
    got = layer_gemms(snip, X, W, dY, entry, snip.OUT_FP32)
    want = oracle_gemms(X, W, dY, entry)
    for g, w in zip(got, want):
        assert np.array_equal(host(g).astype(np.float64), w)


def test_strided_output_and_untouched_padding():
    snip = require_gpu()
    rng = np.random.default_rng(42)
    X = wl.f32_to_bf16_bits(rng.standard_normal((96, 256)).astype(np.float32))
    W = wl.f32_to_bf16_bits(rng.standard_normal((72, 256)).astype(np.float32))
    xq = snip.snip_quantize(to_dev(X), snip.FP8, snip.ROW)
    wq = snip.snip_quantize(to_dev(W), snip.FP8, snip.ROW)
    buf = torch.full((96, 80), 7.0, dtype=torch.float32, device="cuda")
    snip.snip_gemm_fwd((0,) * 6, xq, wq, out=buf[:, :72], out_dtype=snip.OUT_FP32)
    torch.cuda.synchronize()
    want = oracle.gemm_fwd(oracle.fake_quant(X, 0), oracle.fake_quant(W, 0))
    assert rel_fro(host(buf[:, :72]).astype(np.float64), want) <= TOL_F32
    assert torch.all(buf[:, 72:] == 7.0)


def test_error_codes():
    snip = require_gpu()
    xq = snip.alloc_qtensor(64, 128, snip.FP8)
    wq = snip.alloc_qtensor(64, 256, snip.FP8)
    with pytest.raises(snip.SnipError) as e:
        snip.snip_gemm_fwd((0,) * 6, xq, wq)
    assert e.value.status == 4          # contraction extents differ
    wq4 = snip.alloc_qtensor(64, 128, snip.FP4)
    with pytest.raises(snip.SnipError) as e:
        snip.snip_gemm_fwd((0,) * 6, xq, wq4)
    assert e.value.status == 3          # operand format differs from the plan
    x = torch.zeros((32, 48), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(snip.SnipError) as e:
        snip.snip_quantize(x, snip.FP8, snip.ROW, out=snip.alloc_qtensor(32, 64, snip.FP8))
    assert e.value.status == 2


@pytest.mark.parametrize("fa,fb", [(0, 0), (1, 1), (0, 1)])
def test_tiles_agree_bit_for_bit_and_the_launcher_takes_one_of_them(fa, fb, monkeypatch):
    """Every output element sums the same products in the same order under either workgroup tile, so the two tiles
    and the launcher's own pick give identical bits: at a shape where the pick is the narrower tile (its tiles fit
    one round of workgroups) and at one where it is the larger."""
    snip = require_gpu()
    rng = np.random.default_rng(4242)
    for (I, J, R) in ((700, 1300, 512), (4200, 4300, 256)):
        a_bits = wl.f32_to_bf16_bits(rng.standard_normal((I, R)).astype(np.float32))
        b_bits = wl.f32_to_bf16_bits(rng.standard_normal((J, R)).astype(np.float32))
        aq, bq = snip.snip_quantize(to_dev(a_bits), fa, snip.ROW), snip.snip_quantize(to_dev(b_bits), fb, snip.ROW)
        plan = snip.make_plan((fa, fb, 0, 0, 0, 0))
        outs = {}
        for tile in ("big", "wide", None):
            if tile is None:
                monkeypatch.delenv("SNIP_GEMM_TILE", raising=False)
            else:
                monkeypatch.setenv("SNIP_GEMM_TILE", tile)
            y, nrm = snip.snip_gemm_fwd_norm(plan, aq, bq, out_dtype=1)
            torch.cuda.synchronize()
            outs[tile] = (host(y), host(nrm))
        assert np.array_equal(outs["big"][0], outs["wide"][0])
        assert np.array_equal(outs[None][0], outs["big"][0])
        want = oracle.gemm_fwd(oracle.fake_quant(a_bits, fa, oracle.ROW), oracle.fake_quant(b_bits, fb, oracle.ROW))
        assert rel_fro(outs[None][0].astype(np.float64), want) <= TOL_F32
        for t in outs:
            assert float(outs[t][1][0]) == pytest.approx(float((outs[t][0].astype(np.float64) ** 2).sum()), rel=5e-6)


@pytest.mark.parametrize("fmt", [0, 1])
def test_persistent_launch_is_deterministic(fmt):
    """More tiles than compute units (workgroups walk several tiles, the next tile's operands are fetched while
    the current one finishes): two launches give the same bits, with and without the output norm."""
    snip = require_gpu()
    rng = np.random.default_rng(77 + fmt)
    I, J, R = 4700, 4504, 512                # 19 x 18 (or 19 x 36) tiles on 256 compute units, ragged edges
    a_bits = wl.f32_to_bf16_bits(rng.standard_normal((I, R)).astype(np.float32))
    b_bits = wl.f32_to_bf16_bits(rng.standard_normal((J, R)).astype(np.float32))
    aq, bq = snip.snip_quantize(to_dev(a_bits), fmt, snip.ROW), snip.snip_quantize(to_dev(b_bits), fmt, snip.ROW)
    plan = snip.make_plan((fmt, fmt, 0, 0, 0, 0))
    y1 = snip.snip_gemm_fwd(plan, aq, bq)
    y2, n2 = snip.snip_gemm_fwd_norm(plan, aq, bq)
    y3, n3 = snip.snip_gemm_fwd_norm(plan, aq, bq)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2) and torch.equal(y2, y3) and torch.equal(n2, n3)
    rows = rng.choice(I, 64, replace=False)
    want = oracle.gemm_fwd(oracle.fake_quant(a_bits[rows], fmt, oracle.ROW), oracle.fake_quant(b_bits, fmt, oracle.ROW))
    assert rel_fro(host_bf16_as_f64(y1[torch.as_tensor(rows, device="cuda")]), want) <= TOL_BF16
