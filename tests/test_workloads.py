"""Host-side checks of the seeded input generators and plans."""
import numpy as np
import torch

from paper_2602_01410_amd import workloads as wl


def test_bf16_rounding_matches_torch():
    rng = np.random.default_rng(1)
    a = (rng.standard_normal(20000) * 10.0 ** rng.integers(-30, 30, size=20000)).astype(np.float32)
    a[:4] = [0.0, -0.0, np.inf, -np.inf]
    ref = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(wl.f32_to_bf16_bits(a), ref)
    assert np.array_equal(wl.bf16_bits_to_f32(ref), torch.from_numpy(a).to(torch.bfloat16).float().numpy())


def test_draws_are_seeded_and_sliceable():
    a = wl.draw_bf16(42, 3000, 2048, "normal", 0.02)
    b = wl.draw_bf16(42, 3000, 2048, "normal", 0.02)
    assert np.array_equal(a, b)
    part = wl.draw_bf16(42, 3000, 2048, "normal", 0.02, row_start=2040, row_stop=2300)
    assert np.array_equal(part, a[2040:2300])
    assert not np.array_equal(a, wl.draw_bf16(43, 3000, 2048, "normal", 0.02))
    std = wl.bf16_bits_to_f32(a).std()
    assert 0.019 < std < 0.021


def test_outlier_columns_and_heavy_tails():
    a = wl.bf16_bits_to_f32(wl.draw_bf16(7, 512, 1024, "normal_outliers", 1.0))
    col_std = a.std(axis=0)
    assert (col_std > 10).sum() == 1024 // 100
    t = wl.bf16_bits_to_f32(wl.draw_bf16(8, 512, 1024, "student_t3", 1.0))
    assert np.abs(t).max() > 15            # df = 3 tails


def test_config_shapes_and_flops():
    assert wl.CONFIGS[1].flops() == 3 * 2 * 256 * 512 * 512
    assert abs(wl.CONFIGS[2].flops() / 1.649e12 - 1) < 1e-3
    assert abs(wl.CONFIGS[3].flops() / 4.948e12 - 1) < 1e-3
    assert abs(wl.CONFIGS[4].flops() / 1.989e13 - 1) < 1e-3
    assert abs(wl.CONFIGS[5].flops() / 4.206e13 - 1) < 1e-3
    lay = wl.make_layer(wl.CONFIGS[1])
    assert lay.X["x"].shape == (256, 512) and lay.W["lin"].shape == (512, 512)
    assert lay.dY["lin"].shape == (256, 512) and lay.X["x"].dtype == np.uint16


def test_plans():
    cfg = wl.CONFIGS[4]
    assert wl.plan_fp4_fraction(cfg, wl.make_plan(cfg, "fp4")) == 1.0
    assert wl.plan_fp4_fraction(cfg, wl.make_plan(cfg, "fp8")) == 0.0
    mix = wl.make_plan(cfg, "mix50")
    assert mix == wl.make_plan(cfg, "mix50") and 0.0 < wl.plan_fp4_fraction(cfg, mix) < 1.0
    for e in mix:
        assert e[0] == e[1] and e[2] == e[3] and e[4] == e[5]
    tp = wl.make_plan(cfg, "tensor")
    for e in tp:
        assert e[0] == e[5] and e[1] == e[3] and e[2] == e[4]
    assert abs(wl.plan_peak_flops(cfg, wl.make_plan(cfg, "fp4"), 10.0, 5.0) - 10.0) < 1e-9
    assert abs(wl.plan_peak_flops(cfg, wl.make_plan(cfg, "fp8"), 10.0, 5.0) - 5.0) < 1e-9
    assert 5.0 < wl.plan_peak_flops(cfg, mix, 10.0, 5.0) < 10.0
