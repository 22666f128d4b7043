"""Pins for the oracle's AdamW sensitivity factor and weight-divergence estimate (Sec. 4.3.2)."""
import math
from fractions import Fraction

import numpy as np

import oracle


def test_sensitivity_is_the_derivative_of_the_update_direction():
    """The collected term is d/dg of h(g) = m(g) / (sqrt(v(g)) + eps) with m = b1 m' + (1-b1) g and
    v = b2 v' + (1-b2) g^2.  Check it element by element against a central difference of h evaluated in
    exact rational arithmetic around sqrt (high-precision decimal), i.e. without using the closed form."""
    from decimal import Decimal, getcontext
    getcontext().prec = 60
    rng = np.random.default_rng(100)
    b1, b2, eps = 0.9, 0.999, 1e-8
    for _ in range(25):
        m0, g = (float(x) for x in rng.standard_normal(2) * 1e-3)
        v0 = float(abs(rng.standard_normal()) * 1e-6 + 1e-9)

        def h(gd):
            md = Decimal(b1) * Decimal(m0) + (1 - Decimal(b1)) * gd
            vd = Decimal(b2) * Decimal(v0) + (1 - Decimal(b2)) * gd * gd
            return md / (vd.sqrt() + Decimal(eps))

        step = Decimal(10) ** -12
        deriv = (h(Decimal(g) + step) - h(Decimal(g) - step)) / (2 * step)
        m = b1 * m0 + (1 - b1) * g
        v = b2 * v0 + (1 - b2) * g * g
        got = oracle.adamw_sensitivity_sq([m], [v], [g], b1, b2, eps)
        assert math.isclose(math.sqrt(got), abs(float(deriv)), rel_tol=1e-9)


def test_sensitivity_closed_forms():
    n = 1000
    # no first moment: only the first part, constant v
    got = oracle.adamw_sensitivity_sq(np.zeros(n), np.full(n, 4.0), np.ones(n), 0.9, 0.999, 0.5)
    assert math.isclose(got, n * (0.1 / 2.5) ** 2, rel_tol=1e-12)
    # eps = 0, v = 1, m = g = 1: (1-b1) - (1-b2) = b2 - b1
    got = oracle.adamw_sensitivity_sq(np.ones(n), np.ones(n), np.ones(n), 0.5, 0.75, 0.0)
    assert got == n * 0.25 ** 2
    # the sign of m g matters: opposite signs add the two parts
    got = oracle.adamw_sensitivity_sq([-1.0], [1.0], [1.0], 0.5, 0.75, 0.0)
    assert got == 0.75 ** 2
    # v = 0 (an element AdamW never touched): first part alone, 1-b1 over eps
    got = oracle.adamw_sensitivity_sq([0.0], [0.0], [0.0], 0.9, 0.999, 1e-3)
    assert math.isclose(got, (0.1 / 1e-3) ** 2, rel_tol=1e-12)
    assert oracle.adamw_sensitivity_sq([], [], [], 0.9, 0.999, 1e-8) == 0.0
    # additivity over elements
    rng = np.random.default_rng(101)
    m, g = rng.standard_normal(64) * 1e-3, rng.standard_normal(64) * 1e-3
    v = rng.random(64) * 1e-6 + 1e-8
    whole = oracle.adamw_sensitivity_sq(m, v, g, 0.9, 0.999, 1e-8)
    parts = sum(oracle.adamw_sensitivity_sq(m[i:i + 16], v[i:i + 16], g[i:i + 16], 0.9, 0.999, 1e-8) for i in range(0, 64, 16))
    assert math.isclose(whole, parts, rel_tol=1e-13)


def test_sensitivity_scaling_law():
    """Scaling m, g by c and v by c^2 (the same training run at a different loss scale) with eps = 0 scales
    the term by 1/c."""
    rng = np.random.default_rng(102)
    m, g = rng.standard_normal(200), rng.standard_normal(200)
    v = rng.random(200) + 0.1
    base = oracle.adamw_sensitivity_sq(m, v, g, 0.9, 0.99, 0.0)
    c = 1.0 / 1024
    assert math.isclose(oracle.adamw_sensitivity_sq(m * c, v * c * c, g * c, 0.9, 0.99, 0.0), base / (c * c), rel_tol=1e-12)


def test_weight_divergence_closed_forms():
    # t -> infinity: bias corrections vanish
    got = oracle.weight_divergence(1e-3, 0.9, 0.999, 10 ** 7, 16.0, 9.0, 4, 9)
    assert math.isclose(got, 1e-3 * 4.0 * 3.0 / 6.0, rel_tol=1e-12)
    # t = 1: sqrt(1-b2) / (1-b1)
    got = oracle.weight_divergence(2.0, 0.5, 0.75, 1, 1.0, 1.0, 1, 1)
    assert math.isclose(got, 2.0 * 0.5 / 0.5, rel_tol=1e-15)
    # linear in alpha and in each norm
    a = oracle.weight_divergence(1.0, 0.9, 0.99, 5, 2.0, 3.0, 7, 11)
    assert math.isclose(oracle.weight_divergence(3.0, 0.9, 0.99, 5, 2.0 * 4, 3.0 * 9, 7, 11), a * 3 * 2 * 3, rel_tol=1e-14)
    assert math.isclose(oracle.weight_divergence(1.0, 0.9, 0.99, 5, 2.0, 3.0, 28, 11), a / 2, rel_tol=1e-14)
