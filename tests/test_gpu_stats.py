"""GPU parity: snip_quant_error_stats against the CPU oracle, 1e-5 relative."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_01410_amd import workloads as wl

from gpu_util import host, require_gpu, to_dev

pytestmark = pytest.mark.gpu
TOL = 1e-5


def run(snip, bits, axis, rule, per_line=True):
    x = to_dev(bits)
    L = bits.shape[0] if axis == oracle.ROW else bits.shape[1]
    pl = torch.empty((L, 3), dtype=torch.float32, device="cuda") if per_line else None
    out = snip.snip_quant_error_stats(x, axis, rule, per_line=pl)
    torch.cuda.synchronize()
    return host(out), (host(pl) if per_line else None)


@pytest.mark.parametrize("axis", [oracle.ROW, oracle.COL])
@pytest.mark.parametrize("rule", [oracle.NO_OVERFLOW, oracle.FLOOR])
def test_stats_ragged(axis, rule):
    snip = require_gpu()
    rng = np.random.default_rng(30 + axis)
    rows, cols = (200, 2592) if axis == oracle.ROW else (416, 1336)
    a = rng.standard_t(3, size=(rows, cols)) * 10.0 ** rng.integers(-3, 3, size=(rows, 1))
    bits = wl.f32_to_bf16_bits(a.astype(np.float32))
    got, got_lines = run(snip, bits, axis, rule)
    want, want_lines = oracle.stats(bits, axis, rule, per_line=True)
    np.testing.assert_allclose(got, want, rtol=TOL)
    np.testing.assert_allclose(got_lines, want_lines, rtol=TOL, atol=0)


def test_stats_config1_all_tensors():
    snip = require_gpu()
    lay = wl.make_layer(wl.CONFIGS[1])
    for bits in (lay.X["x"], lay.W["lin"], lay.dY["lin"]):
        for axis in (oracle.ROW, oracle.COL):
            got, _ = run(snip, bits, axis, oracle.NO_OVERFLOW, per_line=False)
            np.testing.assert_allclose(got, oracle.stats(bits, axis), rtol=TOL)


def test_stats_zero_on_representable_and_match_fused():
    snip = require_gpu()
    rng = np.random.default_rng(31)
    vals = rng.choice(np.array([0, .5, 1, 1.5, 2, 3, 4, 6.0]), size=(64, 256)) * rng.choice([-1.0, 1.0], size=(64, 256))
    vals *= 2.0 ** rng.integers(-8, 8, size=(64, 1))
    bits = wl.f32_to_bf16_bits(vals.astype(np.float32))
    got, _ = run(snip, bits, oracle.ROW, oracle.NO_OVERFLOW, per_line=False)
    # the error norms are exactly zero; the norm of x itself is an fp32 sum over rows of very different
    # magnitude, so it is held to the tolerance of the statistics, not to equality
    assert got[1] == 0.0 and got[2] == 0.0
    assert got[0] == pytest.approx(np.sum(vals ** 2), rel=TOL)
    # fused (quantize + stats) equals stand-alone for the chosen format
    bits2 = wl.f32_to_bf16_bits(rng.standard_normal((256, 512)).astype(np.float32))
    alone, _ = run(snip, bits2, oracle.COL, oracle.NO_OVERFLOW, per_line=False)
    for fmt, k in ((snip.FP4, 1), (snip.FP8, 2)):
        st = snip.alloc_stats()
        snip.snip_quantize(to_dev(bits2), fmt, snip.COL, stats=st)
        torch.cuda.synchronize()
        f = host(st)
        np.testing.assert_allclose([f[0], f[k]], [alone[0], alone[k]], rtol=1e-6)


def test_stats_deterministic_and_empty():
    snip = require_gpu()
    rng = np.random.default_rng(32)
    bits = wl.f32_to_bf16_bits(rng.standard_normal((512, 1024)).astype(np.float32))
    a, _ = run(snip, bits, oracle.ROW, oracle.NO_OVERFLOW, per_line=False)
    b, _ = run(snip, bits, oracle.ROW, oracle.NO_OVERFLOW, per_line=False)
    assert a.tobytes() == b.tobytes()
    x = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    out = snip.snip_quant_error_stats(x, snip.ROW)
    torch.cuda.synchronize()
    assert host(out).tolist() == [0.0, 0.0, 0.0]


@pytest.mark.parametrize("fill", [0x00, 0xFF, "random"])
def test_stats_workspace_needs_no_initialisation_and_is_reusable(fill):
    """Whatever bytes the workspace holds before the first call, and across calls of different kernels
    and grid shapes that share it, the results stay right."""
    snip = require_gpu()
    rng = np.random.default_rng(33)
    shapes = [(512, 1024), (96, 4096), (2048, 256)]
    tensors = [wl.f32_to_bf16_bits(rng.standard_normal(s).astype(np.float32)) for s in shapes]
    ws = snip.alloc_workspace(2048, 4096)
    if fill == "random":
        ws.copy_(torch.from_numpy(rng.integers(0, 256, size=ws.numel(), dtype=np.uint8)).cuda())
    else:
        ws.fill_(fill)
    for rep in range(2):
        for bits in tensors:
            x = to_dev(bits)
            for axis in (oracle.ROW, oracle.COL):
                want = oracle.stats(bits, axis)
                out = snip.snip_quant_error_stats(x, axis, workspace=ws)
                st = snip.alloc_stats()
                snip.snip_quantize(x, snip.FP4, axis, stats=st, workspace=ws)
                torch.cuda.synchronize()
                np.testing.assert_allclose(host(out), want, rtol=TOL)
                f = host(st)
                np.testing.assert_allclose(f[:2], want[:2], rtol=TOL)
                assert np.isnan(f[2])


@pytest.mark.parametrize("rule", [oracle.NO_OVERFLOW, oracle.FLOOR])
@pytest.mark.parametrize("shape", [(96, 160), (416, 1344), (2048, 4096)])
def test_stats_both_directions_from_one_read(rule, shape):
    """snip_quant_error_stats_both against the oracle's two single-direction results."""
    snip = require_gpu()
    rng = np.random.default_rng(35)
    a = rng.standard_t(3, size=shape) * 10.0 ** rng.integers(-3, 3, size=(shape[0], 1))
    bits = wl.f32_to_bf16_bits(a.astype(np.float32))
    got_r, got_c = snip.snip_quant_error_stats_both(to_dev(bits), rule)
    torch.cuda.synchronize()
    np.testing.assert_allclose(host(got_r), oracle.stats(bits, oracle.ROW, rule), rtol=TOL)
    np.testing.assert_allclose(host(got_c), oracle.stats(bits, oracle.COL, rule), rtol=TOL)


def test_stats_both_special_cases():
    snip = require_gpu()
    rng = np.random.default_rng(36)
    # representable values: both directions report zero error
    vals = rng.choice(np.array([0, .5, 1, 1.5, 2, 3, 4, 6.0]), size=(64, 256)) * rng.choice([-1.0, 1.0], size=(64, 256))
    bits = wl.f32_to_bf16_bits(vals.astype(np.float32))
    r, c = snip.snip_quant_error_stats_both(to_dev(bits))
    torch.cuda.synchronize()
    assert host(r)[1] == 0.0 and host(r)[2] == 0.0 and host(c)[1] == 0.0 and host(c)[2] == 0.0
    assert host(r)[0] == pytest.approx(float((vals ** 2).sum()), rel=TOL)
    # equals the two single-direction calls of the library itself, and is deterministic
    bits = wl.f32_to_bf16_bits(rng.standard_normal((512, 640)).astype(np.float32))
    x = to_dev(bits)
    r1, c1 = snip.snip_quant_error_stats_both(x)
    r2, c2 = snip.snip_quant_error_stats_both(x)
    sr = snip.snip_quant_error_stats(x, snip.ROW)
    sc = snip.snip_quant_error_stats(x, snip.COL)
    torch.cuda.synchronize()
    assert torch.equal(r1, r2) and torch.equal(c1, c2)
    np.testing.assert_allclose(host(r1), host(sr), rtol=1e-6)
    np.testing.assert_allclose(host(c1), host(sc), rtol=1e-6)
    # empty
    e = torch.empty((0, 64), dtype=torch.bfloat16, device="cuda")
    r, c = snip.snip_quant_error_stats_both(e)
    torch.cuda.synchronize()
    assert host(r).tolist() == [0.0, 0.0, 0.0] and host(c).tolist() == [0.0, 0.0, 0.0]


@pytest.mark.parametrize("shift", [-40, 40])
def test_stats_at_the_ends_of_the_documented_magnitude_range(shift):
    """Tensors scaled by 2^-40 and 2^40: differences stay exact and the fp32 squares stay normal, so the
    statistics keep their tolerance against the oracle's fp64 sums (both directions, one-read variant too)."""
    snip = require_gpu()
    rng = np.random.default_rng(33)
    a = rng.standard_normal((256, 640)) * 2.0 ** shift
    bits = wl.f32_to_bf16_bits(a.astype(np.float32))
    for axis in (oracle.ROW, oracle.COL):
        got, got_lines = run(snip, bits, axis, oracle.NO_OVERFLOW)
        want, want_lines = oracle.stats(bits, axis, oracle.NO_OVERFLOW, per_line=True)
        np.testing.assert_allclose(got, want, rtol=TOL)
        np.testing.assert_allclose(got_lines, want_lines, rtol=TOL, atol=0)
    r, c = snip.snip_quant_error_stats_both(to_dev(bits))
    torch.cuda.synchronize()
    np.testing.assert_allclose(host(r), oracle.stats(bits, oracle.ROW), rtol=TOL)
    np.testing.assert_allclose(host(c), oracle.stats(bits, oracle.COL), rtol=TOL)
