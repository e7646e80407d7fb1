"""Pins for the significance function and the intermediate-weight coefficients.

Facts used (Section "I-TiMePReSt", Eq. 1-2; Appendix A.1-A.2): f(0)=1,
f in (0,1], f decreasing to 0, f is the n->infinity limit of (1-lambda*delta/n)^n,
the coefficient 2-1/f lies in (-inf, 1], equals 1 only without staleness and
changes sign where lambda*delta = ln 2.
"""
import math

import numpy as np
import pytest

from oracle import significance as sg


def test_f_endpoints_and_monotone():
    assert sg.f(0, 0.3) == 1.0
    prev = 1.0
    for d in range(1, 200):
        cur = sg.f(d, 0.3)
        assert 0.0 < cur < prev <= 1.0
        prev = cur
    assert sg.f(10_000, 0.3) < 1e-300 or sg.f(10_000, 0.3) == 0.0 or sg.f(10_000, 0.3) < 1e-12


@pytest.mark.parametrize("lam,delta", [(0.01, 1), (0.1, 3), (math.log(2), 1), (1.0, 2)])
def test_f_is_limit_of_compound_decay(lam, delta):
    # independent evaluation of the limit: the product of n equal decay steps
    n = 10**6
    assert abs(sg.f_finite(delta, lam, n) - sg.f(delta, lam)) < 1e-5
    # and the defining differential property: f' = -lambda f  (central difference)
    h = 1e-5
    d = (sg.f(delta + h, lam) - sg.f(delta - h, lam)) / (2 * h)
    assert abs(d + lam * sg.f(delta, lam)) < 1e-8


def test_f_difference_equation():
    # Appendix A.1: f(delta + d) = f(delta) * (1 - lambda*d) to first order in d
    lam, d = 0.2, 1e-6
    for delta in (0.0, 1.0, 2.5):
        lhs = sg.f(delta + d, lam)
        rhs = sg.f(delta, lam) * (1 - lam * d)
        assert abs(lhs - rhs) < 1e-11


def test_eq1_coefficient_range_and_zero():
    lam = 0.1
    assert sg.coefficients("eq1", 0, lam) == (1.0, 0.0)
    for d in range(1, 100):
        a, b = sg.coefficients("eq1", d, lam)
        assert b == 0.0 and a < 1.0
    # zero exactly where lambda*delta = ln 2, negative beyond
    a, _ = sg.coefficients("eq1", 1, math.log(2))
    assert abs(a) < 1e-15
    assert sg.coefficients("eq1", 2, math.log(2))[0] < 0
    # written out independently: 2 - e^{lambda delta}
    for d in (1, 2, 3):
        assert abs(sg.coefficients("eq1", d, 0.37)[0] - (2 - math.e ** (0.37 * d))) < 1e-14


def test_convex_coefficients():
    assert sg.coefficients("convex", 0, 0.5) == (1.0, 0.0)
    a, b = sg.coefficients("convex", 1, math.log(2))
    assert abs(a - 0.5) < 1e-15 and abs(b - 0.5) < 1e-15
    for d in range(0, 50):
        a, b = sg.coefficients("convex", d, 0.1)
        assert 0 < a <= 1 and 0 <= b < 1 and abs(a + b - 1) < 1e-15
    a, b = sg.coefficients("convex", 10_000, 0.1)
    assert a < 1e-12 and abs(b - 1) < 1e-12


def test_fixed_policies_ignore_delta():
    for d in (0, 1, 7):
        assert sg.coefficients("latest", d, 0.1) == (0.0, 1.0)
        assert sg.coefficients("stashed", d, 0.1) == (1.0, 0.0)


def test_appendix_a2_algebra():
    # Appendix A.2 solves  W = f*S + (1-f)*(W - S)  for W; the solution is (2 - 1/f) S.
    rng = np.random.default_rng(0)
    S = rng.standard_normal(16)
    for d in (1, 2, 3):
        fd = sg.f(d, 0.1)
        W = sg.coefficients("eq1", d, 0.1)[0] * S
        assert np.allclose(W, fd * S + (1 - fd) * (W - S), rtol=0, atol=1e-13)
