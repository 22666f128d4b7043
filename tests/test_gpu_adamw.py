"""GPU parity: the AdamW sensitivity factor (Sec. 4.3.2) against the CPU oracle.

Tolerance 1e-5 relative: each element's term carries a few fp32 roundings (square root, two divisions, a
handful of products: ~5e-7 relative, the second part is ~1 % of the first for AdamW's betas so nothing
cancels), squares are added per lane and wave in fp32 (~1e-6) and across waves in double."""
import numpy as np
import pytest
import torch

import oracle
from paper_2602_01410_amd import workloads as wl

from gpu_util import host, require_gpu

pytestmark = pytest.mark.gpu
TOL = 1e-5
B1, B2, EPS = float(np.float32(0.9)), float(np.float32(0.999)), float(np.float32(1e-8))


def run(snip, m, v, g, b1=B1, b2=B2, eps=EPS):
    out = snip.snip_adamw_sensitivity(torch.from_numpy(m).cuda(), torch.from_numpy(v).cuda(), g.cuda(), b1, b2, eps)
    torch.cuda.synchronize()
    return float(host(out)[0])


@pytest.mark.parametrize("n", [0, 1, 3, 4, 1000, 262144 + 5, 3 * 1024 * 1024 + 2])
def test_adamw_fp32_gradient_sizes_and_tails(n):
    snip = require_gpu()
    rng = np.random.default_rng(110)
    g = (1e-3 * rng.standard_normal(n)).astype(np.float32)
    m = (0.3e-3 * rng.standard_normal(n)).astype(np.float32)
    v = (1e-6 * (0.5 + rng.random(n))).astype(np.float32)
    got = run(snip, m, v, torch.from_numpy(g))
    want = oracle.adamw_sensitivity_sq(m, v, g, B1, B2, EPS)
    assert got == pytest.approx(want, rel=TOL)


def test_adamw_config_state_bf16_and_fp32_gradient():
    """The optimizer state of config 2's 'gate' weight (8192 x 2048) with the gradient as fp32 and as the
    bf16 tensor a wgrad call would deliver."""
    snip = require_gpu()
    m, v, g = wl.make_optimizer_state(wl.CONFIGS[2], "gate")
    want = oracle.adamw_sensitivity_sq(m, v, g, B1, B2, EPS)
    assert run(snip, m.ravel(), v.ravel(), torch.from_numpy(g.ravel())) == pytest.approx(want, rel=TOL)
    g16 = torch.from_numpy(g.ravel()).to(torch.bfloat16)
    want16 = oracle.adamw_sensitivity_sq(m, v, g16.to(torch.float64).numpy(), B1, B2, EPS)
    assert run(snip, m.ravel(), v.ravel(), g16) == pytest.approx(want16, rel=TOL)


def test_adamw_special_elements_and_determinism():
    """Untouched elements (v = 0), m and g of opposite sign, eps = 0, other betas."""
    snip = require_gpu()
    rng = np.random.default_rng(111)
    n = 50000
    g = (1e-2 * rng.standard_normal(n)).astype(np.float32)
    m = (-np.abs(g) * np.sign(g) * 0.5).astype(np.float32)       # opposite sign to g
    v = (1e-4 * (0.1 + rng.random(n))).astype(np.float32)
    dead = rng.random(n) < 0.1
    g[dead] = 0; m[dead] = 0; v[dead] = 0
    b1, b2, eps = float(np.float32(0.8)), float(np.float32(0.95)), float(np.float32(1e-6))
    a = run(snip, m, v, torch.from_numpy(g), b1, b2, eps)
    b = run(snip, m, v, torch.from_numpy(g), b1, b2, eps)
    assert a == b
    assert a == pytest.approx(oracle.adamw_sensitivity_sq(m, v, g, b1, b2, eps), rel=TOL)
    live = ~dead
    got0 = run(snip, m[live], v[live], torch.from_numpy(g[live]), b1, b2, 0.0)
    assert got0 == pytest.approx(oracle.adamw_sensitivity_sq(m[live], v[live], g[live], b1, b2, 0.0), rel=TOL)


def test_weight_divergence_chain():
    """Sensitivity from the GPU, combined on the host, against the same chain in the oracle."""
    snip = require_gpu()
    cfg = wl.CONFIGS[1]
    lin = cfg.linears[0]
    m, v, g = wl.make_optimizer_state(cfg, lin.name)
    s = run(snip, m.ravel(), v.ravel(), torch.from_numpy(g.ravel()))
    err_g_sq = 1e-9
    got = snip.snip_weight_divergence(3e-4, B1, B2, 1000, s, err_g_sq, lin.N, lin.K)
    want = oracle.weight_divergence(3e-4, B1, B2, 1000, oracle.adamw_sensitivity_sq(m, v, g, B1, B2, EPS), err_g_sq, lin.N, lin.K)
    assert got == pytest.approx(want, rel=TOL)
