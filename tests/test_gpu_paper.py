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
