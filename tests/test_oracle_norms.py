"""Pins for the oracle's output-norm and loss-divergence functions (Sec. 3.1 Step 1: norms of Y, dX, dW;
Sec. 4.2 "Loss Divergence in Forward Pass").  None of these checks re-types the oracle's own formula:
rounding is pinned to tie tables, to torch's and the input generator's fp32->bf16 casts and to exhaustive
idempotence; the norm to closed forms; the estimate to Pythagorean triples, limits and symmetries."""
import math

import numpy as np
import torch

import oracle
from paper_2602_01410_amd import workloads as wl


def test_round_bf16_tie_table():
    cases = [
        (257.0, 256.0),                      # halfway between 256 (even mantissa) and 258
        (259.0, 260.0),                      # halfway between 258 (odd) and 260 (even)
        (1.0 + 2.0 ** -8, 1.0),
        (1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -6),
        (1.0 + 2.0 ** -8 + 2.0 ** -30, 1.0 + 2.0 ** -7),   # just above the tie
        (1.0 + 2.0 ** -8 - 2.0 ** -30, 1.0),               # just below
        (-257.0, -256.0),
        (3.0, 3.0), (0.0, 0.0), (448.0, 448.0),
        (255.5, 256.0),                      # rounds up into the next binade
        (2.0 ** -133, 2.0 ** -133),          # smallest bf16 subnormal
        (2.0 ** -134, 0.0),                  # tie between 0 and 2^-133 -> even
        (1.5 * 2.0 ** -133, 2.0 ** -132),    # tie between 1 and 2 quanta -> even
    ]
    for v, want in cases:
        assert oracle.round_output(v, oracle.OUT_BF16) == want, (v, want)


def test_round_bf16_idempotent_on_every_finite_bf16():
    bits = np.arange(65536, dtype=np.uint32)
    f32 = (bits << 16).astype(np.uint32).view(np.float32)
    vals = f32[np.isfinite(f32)].astype(np.float64)
    got = np.array([oracle.round_output(v) for v in vals])
    assert np.array_equal(got, vals)


def test_round_bf16_matches_torch_and_generator_casts():
    rng = np.random.default_rng(50)
    x = (rng.standard_normal(20000) * 10.0 ** rng.integers(-20, 20, size=20000)).astype(np.float32)
    got = np.array([oracle.round_output(float(v)) for v in x])
    t = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    g = wl.bf16_bits_to_f32(wl.f32_to_bf16_bits(x)).astype(np.float64)
    assert np.array_equal(got, t)
    assert np.array_equal(got, g)


def test_round_fp32_is_the_ieee_single_cast():
    rng = np.random.default_rng(51)
    x = rng.standard_normal(5000) * 10.0 ** rng.integers(-30, 30, size=5000)
    got = np.array([oracle.round_output(float(v), oracle.OUT_FP32) for v in x])
    assert np.array_equal(got, x.astype(np.float32).astype(np.float64))


def test_output_sum_sq_closed_forms():
    M, N, K = 5, 7, 64
    Y = oracle.gemm_fwd(np.ones((M, K)), np.ones((N, K)))
    assert oracle.output_sum_sq(Y) == M * N * K * K
    assert oracle.output_sum_sq(Y, oracle.OUT_FP32) == M * N * K * K
    # elements that the bf16 output cannot hold are rounded before they are squared
    assert oracle.output_sum_sq([257.0, 259.0, 1.0 + 2.0 ** -8]) == 256.0 ** 2 + 260.0 ** 2 + 1.0
    assert oracle.output_sum_sq([257.0, 259.0], oracle.OUT_FP32) == 257.0 ** 2 + 259.0 ** 2
    assert oracle.output_sum_sq([]) == 0.0
    # sign and order do not matter, one-hot picks one square
    assert oracle.output_sum_sq([0, 0, -3.0, 0]) == 9.0


def test_output_sum_sq_against_torch_bf16_route():
    rng = np.random.default_rng(52)
    c = rng.standard_normal((37, 53)).astype(np.float32)        # fp32 values: torch's cast is a single rounding
    want = float((torch.from_numpy(c).to(torch.bfloat16).to(torch.float64) ** 2).sum())
    assert math.isclose(oracle.output_sum_sq(c.astype(np.float64)), want, rel_tol=1e-14)
    want32 = float((c.astype(np.float64) ** 2).sum())
    assert math.isclose(oracle.output_sum_sq(c.astype(np.float64), oracle.OUT_FP32), want32, rel_tol=1e-14)


def test_loss_divergence_pythagorean_and_limits():
    M, N, K = 16, 4, 9
    # terms 3 and 4 -> 5:  |gX||dX|/sqrt(MK) = 3  with MK = 144: |gX||dX| = 36
    gx, ex = 6.0 ** 2, 6.0 ** 2
    # |gW||dW|/sqrt(NK) = 4 with NK = 36: |gW||dW| = 24
    gw, ew = 4.0 ** 2, 6.0 ** 2
    assert math.isclose(oracle.loss_divergence(gx, ex, M, gw, ew, N, K), 5.0, rel_tol=1e-15)
    # one error absent: the other term alone
    assert math.isclose(oracle.loss_divergence(gx, ex, M, gw, 0.0, N, K), 3.0, rel_tol=1e-15)
    assert math.isclose(oracle.loss_divergence(gx, 0.0, M, gw, ew, N, K), 4.0, rel_tol=1e-15)
    assert oracle.loss_divergence(0.0, 0.0, M, 0.0, 0.0, N, K) == 0.0


def test_loss_divergence_homogeneity_and_symmetry():
    rng = np.random.default_rng(53)
    for _ in range(20):
        gx, ex, gw, ew = rng.uniform(0.1, 10.0, size=4)
        M, N, K = (int(v) for v in rng.integers(1, 500, size=3))
        base = oracle.loss_divergence(gx, ex, M, gw, ew, N, K)
        # doubling both error norms (x4 on the squares) doubles the estimate; same for both gradient norms
        assert math.isclose(oracle.loss_divergence(gx, 4 * ex, M, gw, 4 * ew, N, K), 2 * base, rel_tol=1e-14)
        assert math.isclose(oracle.loss_divergence(4 * gx, ex, M, 4 * gw, ew, N, K), 2 * base, rel_tol=1e-14)
        # exchanging the roles of the two operands (and M with N) leaves it unchanged
        assert math.isclose(oracle.loss_divergence(gw, ew, N, gx, ex, M, K), base, rel_tol=1e-14)
        # more tokens at fixed norms dilute the activation term only: M -> 4M halves it
        only_x = oracle.loss_divergence(gx, ex, M, gw, 0.0, N, K)
        assert math.isclose(oracle.loss_divergence(gx, ex, 4 * M, gw, 0.0, N, K), only_x / 2, rel_tol=1e-14)


def test_loss_divergence_from_matrices():
    """Evaluate the estimate from actual small matrices with numpy's norms, term by term."""
    rng = np.random.default_rng(54)
    M, N, K = 6, 5, 32
    dX, dW = rng.standard_normal((M, K)), rng.standard_normal((N, K))
    eX, eW = 0.01 * rng.standard_normal((M, K)), 0.02 * rng.standard_normal((N, K))
    tx = np.linalg.norm(dX) * np.linalg.norm(eX) / math.sqrt(M * K)
    tw = np.linalg.norm(dW) * np.linalg.norm(eW) / math.sqrt(N * K)
    got = oracle.loss_divergence((dX ** 2).sum(), (eX ** 2).sum(), M, (dW ** 2).sum(), (eW ** 2).sum(), N, K)
    assert math.isclose(got, math.hypot(tx, tw), rel_tol=1e-13)
