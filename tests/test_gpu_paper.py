"""GPU parity: the paper's own recipe (real-valued scale FPX_MAX / amax per 1x128 tile or 128x128 block)
against the CPU oracle.  Codes and fp32 scales bit for bit (both sides form the scale and x * scale in fp32
with one rounding each); statistics to 1e-5."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_01410_amd import workloads as wl

from gpu_util import host, require_gpu, to_dev

pytestmark = pytest.mark.gpu

GROUPS = [oracle.TILE_1x128, oracle.BLOCK_128x128]


def data(rng, rows, cols, special=True):
    a = rng.standard_t(3, size=(rows, cols)) * 10.0 ** rng.integers(-6, 6, size=(rows, 1))
    bits = wl.f32_to_bf16_bits(a.astype(np.float32))
    if special:
        bits[1, :128] = 0                                    # an all-zero tile
        bits[2, 5] = 0x7F80                                  # +inf: its group gets a NaN scale and zero codes
        bits[3, 130:140] = np.arange(1, 11, dtype=np.uint16)  # bf16 subnormals among ordinary values
        if rows > 8:
            bits[8, :128] = np.arange(1, 129, dtype=np.uint16) % 3     # a tile of tiny subnormals: capped scale
    return bits


@pytest.mark.parametrize("fmt", [oracle.FP8, oracle.FP4])
@pytest.mark.parametrize("group", GROUPS)
def test_quantize_paper_rows(fmt, group):
    snip = require_gpu()
    rng = np.random.default_rng(130 + fmt)
    bits = data(rng, 301, 1664)                              # rows ragged against 4 and 128, 13 tiles per row
    codes, scales = snip.snip_quantize_paper(to_dev(bits), fmt, snip.ROW, group)
    torch.cuda.synchronize()
    want_c, want_s = oracle.quantize_paper(bits, fmt, oracle.ROW, group)
    assert np.array_equal(host(scales).view(np.uint32), want_s.view(np.uint32))
    assert np.array_equal(host(codes), want_c)


@pytest.mark.parametrize("fmt", [oracle.FP8, oracle.FP4])
@pytest.mark.parametrize("group", GROUPS)
def test_quantize_paper_columns(fmt, group):
    snip = require_gpu()
    rng = np.random.default_rng(132 + fmt)
    bits = data(rng, 384, 1336)                              # three row groups, columns ragged against 128
    codes, scales = snip.snip_quantize_paper(to_dev(bits), fmt, snip.COL, group)
    torch.cuda.synchronize()
    want_c, want_s = oracle.quantize_paper(bits, fmt, oracle.COL, group)
    assert np.array_equal(host(scales).view(np.uint32), want_s.view(np.uint32))
    assert np.array_equal(host(codes), want_c)


@pytest.mark.parametrize("axis", [oracle.ROW, oracle.COL])
@pytest.mark.parametrize("group", GROUPS)
def test_stats_paper(axis, group):
    snip = require_gpu()
    rng = np.random.default_rng(134 + axis)
    rows, cols = (300, 1280) if axis == oracle.ROW else (512, 1096)
    bits = data(rng, rows, cols, special=False)
    out = snip.snip_quant_error_stats_paper(to_dev(bits), axis, group)
    torch.cuda.synchronize()
    np.testing.assert_allclose(host(out), oracle.stats_paper(bits, axis, group), rtol=1e-5)


def test_paper_recipe_on_config_tensors():
    """Activations and gradients with tiles, the weight with blocks (the paper's assignment), config 2's q."""
    snip = require_gpu()
    cfg = wl.CONFIGS[2]
    X = wl.make_tensor(cfg, "X", "attn_in", 0, 512)
    W = wl.make_tensor(cfg, "W", "q")
    for bits, group in ((X, oracle.TILE_1x128), (W, oracle.BLOCK_128x128)):
        for axis in (oracle.ROW, oracle.COL):
            out = snip.snip_quant_error_stats_paper(to_dev(bits), axis, group)
            c, s = snip.snip_quantize_paper(to_dev(bits), snip.FP8, axis, group)
            torch.cuda.synchronize()
            np.testing.assert_allclose(host(out), oracle.stats_paper(bits, axis, group), rtol=1e-5)
            wc, ws = oracle.quantize_paper(bits, oracle.FP8, axis, group)
            assert np.array_equal(host(c), wc) and np.array_equal(host(s).view(np.uint32), ws.view(np.uint32))


def test_paper_validation():
    snip = require_gpu()
    x = torch.zeros((64, 96), dtype=torch.bfloat16, device="cuda")          # 96 is not a multiple of 128
    with pytest.raises(snip.SnipError):
        snip.snip_quantize_paper(x, snip.FP8, snip.ROW, snip.TILE_1x128)
    with pytest.raises(snip.SnipError):
        snip.snip_quant_error_stats_paper(x, snip.COL, snip.TILE_1x128)     # 64 rows: blocked extent not a multiple of 128


def _layer_paper(snip, X, W, dY, fx, fw, fdy, out_dtype):
    """The three GEMMs of a linear with the paper's assignment: tiles for X and dY, blocks for W."""
    T, B = snip.TILE_1x128, snip.BLOCK_128x128
    dX_, dW_, ddY = to_dev(X), to_dev(W), to_dev(dY)
    q = snip.snip_quantize_paper
    xr, wr = q(dX_, fx, snip.ROW, T), q(dW_, fw, snip.ROW, B)
    dyr, wc = q(ddY, fdy, snip.ROW, T), q(dW_, fw, snip.COL, B)
    dyc, xc = q(ddY, fdy, snip.COL, T), q(dX_, fx, snip.COL, T)
    y = snip.snip_gemm_paper(*xr, fx, T, *wr, fw, B, out_dtype=out_dtype)
    dx = snip.snip_gemm_paper(*dyr, fdy, T, *wc, fw, B, out_dtype=out_dtype)
    dw = snip.snip_gemm_paper(*dyc, fdy, T, *xc, fx, T, out_dtype=out_dtype)
    torch.cuda.synchronize()
    return y, dx, dw


def _oracle_layer_paper(X, W, dY, fx, fw, fdy):
    T, B = oracle.TILE_1x128, oracle.BLOCK_128x128
    def dq(bits, fmt, axis, group):
        c, s = oracle.quantize_paper(bits, fmt, axis, group)
        return oracle.dequantize_paper(c, s, fmt, group)
    # all three products have the form C[i][j] = sum_r A[i][r] B[j][r] on the stored matrices
    y = oracle.gemm_fwd(dq(X, fx, oracle.ROW, T), dq(W, fw, oracle.ROW, B))
    dx = oracle.gemm_fwd(dq(dY, fdy, oracle.ROW, T), dq(W, fw, oracle.COL, B))
    dw = oracle.gemm_fwd(dq(dY, fdy, oracle.COL, T), dq(X, fx, oracle.COL, T))
    return y, dx, dw


@pytest.mark.parametrize("fmts", [(0, 0, 0), (1, 1, 1), (0, 0, 1), (1, 0, 1)])
@pytest.mark.parametrize("out_dtype", [0, 1])
def test_gemm_paper_layer(fmts, out_dtype):
    """M, N, K multiples of 128 (every one of them is a contraction extent of one of the three GEMMs) but
    not of each other; several tiles per output dimension."""
    snip = require_gpu()
    fx, fw, fdy = fmts
    rng = np.random.default_rng(140)
    M, N, K = 384, 256, 640
    X = wl.f32_to_bf16_bits(rng.standard_t(3, size=(M, K)).astype(np.float32))
    W = wl.f32_to_bf16_bits((0.02 * rng.standard_normal((N, K))).astype(np.float32))
    dY = wl.f32_to_bf16_bits((1e-3 * rng.standard_normal((M, N)) * 10.0 ** rng.integers(-2, 2, size=(M, 1))).astype(np.float32))
    got = _layer_paper(snip, X, W, dY, fx, fw, fdy, out_dtype)
    want = _oracle_layer_paper(X, W, dY, fx, fw, fdy)
    tol = 2e-3 if out_dtype == 0 else 1e-4
    for g, w in zip(got, want):
        gg = host(g.to(torch.float64))
        assert np.linalg.norm(gg - w) <= tol * np.linalg.norm(w)


def test_gemm_paper_ragged_outputs_and_exact_case():
    """Output extents that are not multiples of the 128 x 128 tile, and a case where everything is exact:
    grid-valued operands with the type's maximum in every group, so scales are powers of two and the
    product of small integers needs no rounding."""
    snip = require_gpu()
    rng = np.random.default_rng(141)
    I, J, R = 200, 72, 256
    T = snip.TILE_1x128
    vals = np.array([-6, -4, -3, -2, -1.5, -1, -.5, 0, .5, 1, 1.5, 2, 3, 4, 6.0])
    def draw(r):
        a = rng.choice(vals, size=(r, R))
        a[:, 0] = 6.0; a[:, 128] = -6.0
        a *= 2.0 ** rng.integers(-2, 3, size=(r, 1))
        return wl.f32_to_bf16_bits(a.astype(np.float32))
    A, B = draw(I), draw(J)
    qa = snip.snip_quantize_paper(to_dev(A), snip.FP4, snip.ROW, T)
    qb = snip.snip_quantize_paper(to_dev(B), snip.FP4, snip.ROW, T)
    c = snip.snip_gemm_paper(*qa, snip.FP4, T, *qb, snip.FP4, T, out_dtype=snip.OUT_FP32)
    torch.cuda.synchronize()
    a64 = wl.bf16_bits_to_f32(A).astype(np.float64)
    b64 = wl.bf16_bits_to_f32(B).astype(np.float64)
    assert np.array_equal(host(c).astype(np.float64), a64 @ b64.T)
