"""Pins for the oracle's marginal gains and hit utility (CPU only).

Every check compares the oracle with something it does not compute itself:
exact rational arithmetic, closed forms, quadrature of the posterior, a
log-gamma Beta ratio.  Citations: Sec. 3.2 Eq. 3 / Eq. 5, App. A.
"""
from fractions import Fraction
from math import comb

import numpy as np
import pytest
from scipy import integrate, special

ULP = 2.0 ** -52


def exact_gain(a: Fraction, b: Fraction, l: int) -> Fraction:
    """B(a+1, b+l)/B(a, b) = a * (b)_l / (a+b)_{l+1} with rising factorials."""
    num = a
    for k in range(l):
        num *= b + k
    den = Fraction(1)
    for k in range(l + 1):
        den *= a + b + k
    return num / den


def exact_utility(a: Fraction, b: Fraction, d: int) -> Fraction:
    """1 - B(a, b+d)/B(a, b) = 1 - prod_{k<d} (b+k)/(a+b+k)."""
    e = Fraction(1)
    for k in range(d):
        e *= (b + k) / (a + b + k)
    return 1 - e


@pytest.mark.parametrize("g0", [1, 2, 4, 8, 16])
def test_gains_match_exact_rationals(oracle, g0):
    L = 200
    for c in range(g0 + 1):
        a, b = Fraction(1 + c), Fraction(1 + g0 - c)
        got = oracle.marginal_gains(float(a), float(b), L)
        for l in range(L):
            want = exact_gain(a, b, l)
            err = abs(Fraction(got[l]) - want) / want
            # two roundings per step of the recurrence
            assert err <= (2 * l + 1) * ULP, (g0, c, l, float(err))


def test_gains_closed_form_c0(oracle):
    # c = 0, uniform prior: alpha = 1, beta = G0+1:  M(l) = (G0+1)/((G0+1+l)(G0+2+l))
    for g0 in (2, 4, 8, 32):
        got = oracle.marginal_gains(1.0, g0 + 1.0, 300)
        l = np.arange(300, dtype=np.float64)
        want = (g0 + 1.0) / ((g0 + 1.0 + l) * (g0 + 2.0 + l))
        np.testing.assert_allclose(got, want, rtol=1e-13, atol=0)


def test_gains_strictly_decreasing_positive_and_ratio(oracle):
    rng = np.random.default_rng(5)
    cases = [(1.0 + c, 1.0 + g0 - c) for g0 in (2, 4, 8, 16) for c in range(g0 + 1)]
    cases += [(float(a), float(b)) for a, b in zip(rng.uniform(0.01, 20, 50), rng.uniform(0.01, 20, 50))]
    for a, b in cases:
        m = oracle.marginal_gains(a, b, 2000)
        assert np.all(m > 0)
        assert np.all(np.diff(m) < 0), (a, b)          # strict even after rounding
        l = np.arange(1999, dtype=np.float64)
        np.testing.assert_allclose(m[1:] / m[:-1], (b + l) / (a + b + l + 1), rtol=1e-14)
        assert m[0] == a / (a + b)


def test_first_gain_is_posterior_mean(oracle):
    # M(0) = E[P] under Beta(alpha, beta)
    for a, b in [(1.0, 5.0), (3.0, 3.0), (0.3, 7.7), (9.0, 1.0)]:
        mean, _ = integrate.quad(lambda p: p * p ** (a - 1) * (1 - p) ** (b - 1), 0, 1)
        mean /= special.beta(a, b)
        assert oracle.marginal_gains(a, b, 1)[0] == pytest.approx(mean, rel=1e-9)


@pytest.mark.parametrize("g0", [2, 4, 8, 16])
def test_utility_closed_forms(oracle, g0):
    for d in range(0, 120):
        # c = 0:  U = d/(G0+1+d)
        assert oracle.hit_utility(1.0, g0 + 1.0, d) == pytest.approx(d / (g0 + 1.0 + d), rel=1e-13, abs=0)
        # c = G0: U = 1 - 1/C(G0+1+d, d)
        want = 1 - Fraction(1, comb(g0 + 1 + d, d))
        assert oracle.hit_utility(g0 + 1.0, 1.0, d) == pytest.approx(float(want), rel=1e-13, abs=1e-300)
    assert oracle.hit_utility(1.0, g0 + 1.0, 0) == 0.0


def test_utility_matches_exact_rationals(oracle):
    for g0 in (2, 4, 8):
        for c in range(g0 + 1):
            a, b = Fraction(1 + c), Fraction(1 + g0 - c)
            for d in (0, 1, 2, 3, 7, 20, 64):
                want = exact_utility(a, b, d)
                got = oracle.hit_utility(float(a), float(b), d)
                assert abs(Fraction(got) - want) <= 4 * (d + 1) * ULP


def test_utility_is_posterior_expectation_by_quadrature(oracle):
    # Eq. 3: U(d) = E[1 - (1-P)^d], P ~ Beta(a, b).  For integer a, b the
    # integrand is a polynomial, so Gauss-Legendre with enough nodes is exact.
    x, w = np.polynomial.legendre.leggauss(80)
    p = 0.5 * (x + 1.0)
    w = 0.5 * w
    for g0 in (4, 8):
        for c in range(g0 + 1):
            a, b = 1 + c, 1 + g0 - c
            dens = p ** (a - 1) * (1 - p) ** (b - 1)
            norm = np.dot(w, dens)
            for d in (1, 2, 5, 17, 40):
                want = np.dot(w, dens * (1 - (1 - p) ** d)) / norm
                assert oracle.hit_utility(float(a), float(b), d) == pytest.approx(want, rel=1e-12)
    # real-valued posteriors (learned prior, App. D): adaptive quadrature
    for a, b in [(0.5, 2.5), (2.3, 0.7), (0.0625, 8.1875), (7.5, 7.5)]:
        for d in (1, 3, 12):
            val, _ = integrate.quad(lambda q: (1 - (1 - q) ** d) * q ** (a - 1) * (1 - q) ** (b - 1),
                                    0, 1, epsabs=0, epsrel=1e-11, limit=400)
            assert oracle.hit_utility(a, b, d) == pytest.approx(val / special.beta(a, b), rel=1e-7)


def test_utility_matches_log_gamma_beta_ratio(oracle):
    for a, b in [(1.0, 9.0), (4.0, 6.0), (9.0, 1.0), (0.4, 3.1), (11.5, 0.5)]:
        for d in (1, 4, 33, 257):
            want = -np.expm1(special.betaln(a, b + d) - special.betaln(a, b))
            assert oracle.hit_utility(a, b, d) == pytest.approx(want, rel=1e-11)


def test_gain_is_utility_increment_and_sums_to_utility(oracle):
    # Eq. 5: M(l) = U(l+1) - U(l);  App. A: U(d) = sum_{l<d} M(l)
    for a, b in [(1.0, 5.0), (3.0, 3.0), (5.0, 1.0), (1.0, 17.0), (0.7, 2.2)]:
        m = oracle.marginal_gains(a, b, 100)
        u = np.array([oracle.hit_utility(a, b, d) for d in range(101)])
        np.testing.assert_allclose(np.diff(u), m, rtol=0, atol=1e-15)
        np.testing.assert_allclose(np.cumsum(m), u[1:], rtol=1e-12, atol=0)


def test_known_exact_ties_between_classes():
    # G0 = 4, uniform prior: M_{c=0}(1) = M_{c=1}(2) = M_{c=4}(1) = 5/42 exactly, and
    # M_c(1) = M_{G0-c}(1) for every c: the allocation problem has exact ties.
    assert exact_gain(Fraction(1), Fraction(5), 1) == Fraction(5, 42)
    assert exact_gain(Fraction(2), Fraction(4), 2) == Fraction(5, 42)
    assert exact_gain(Fraction(5), Fraction(1), 1) == Fraction(5, 42)
    for g0 in (2, 4, 8):
        for c in range(g0 + 1):
            assert exact_gain(Fraction(1 + c), Fraction(1 + g0 - c), 1) == \
                exact_gain(Fraction(1 + g0 - c), Fraction(1 + c), 1)
