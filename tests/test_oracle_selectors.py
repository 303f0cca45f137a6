"""Pins for the oracle's analytic breakpoint selectors and its fixed-(m, p)
error evaluator.

The selectors are the paper's own way of choosing the breakpoint (Section 3.3,
Section 5.1): assume a zero-mean Gaussian or Laplacian truncated to [-m, m],
minimise the expected error of Eq.6 over (0, m/2).  The checks below restate
that with scipy's distribution functions and a dense grid instead of the
oracle's root finder, use the paper's Eq.12 (which holds only at a root of
Eq.11), and compare the Section 5.1 logarithmic fit with the solver.
"""
import math
import os
from fractions import Fraction

import numpy as np
import pytest
from scipy import stats

from oracle import pwlq_ref as R

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _constants():
    out = {}
    with open(os.path.join(GOLD, "paper_constants.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            name, value = line.split()[:2]
            out[name] = float(value)
    return out


def _group_with_moments(m, sigma=None, beta=None, K=4096):
    """A group whose absmax is m and whose root mean square is sigma (or whose
    mean magnitude is beta): one element m, the rest +-c.  The selectors see the
    data only through these statistics."""
    if sigma is not None:
        c = math.sqrt((K * sigma * sigma - m * m) / (K - 1))
    else:
        c = (K * beta - m) / (K - 1)
    assert 0 < c < m
    w = np.full(K, c, np.float64)
    w[1::2] *= -1
    w[0] = m
    return w.astype(np.float32)[None, :]


def _eq6(p, m, cdf):
    """Eq.6 without the factor C(b-1): (m-p)^2 + m (2p-m) [2F(p) - 1]."""
    return (m - p) ** 2 + m * (2 * p - m) * (2 * cdf(p) - 1)


def _truncated(dist, m):
    lo, hi = dist.cdf(-m), dist.cdf(m)
    return (lambda p: (dist.cdf(p) - lo) / (hi - lo)), (lambda p: dist.pdf(p) / (hi - lo))


def _grid_argmin(m, cdf, points=400_001):
    p = np.linspace(0.0, 0.5 * m, points)[1:-1]
    return float(p[np.argmin(_eq6(p, m, cdf))]), 0.5 * m / (points - 1)


@pytest.mark.parametrize("x", [2.0, 3.0, 4.0, 5.0, 6.0, 8.0])
@pytest.mark.parametrize("sigma", [1.0, 0.037])
def test_gaussian_solver_minimises_eq6(x, sigma):
    m = x * sigma
    w = _group_with_moments(m, sigma=sigma)
    s_hat = float(np.sqrt(np.mean(w.astype(np.float64) ** 2)))
    m_hat = float(np.abs(w).max())
    p, m_out = R.select_analytic(w, R.GAUSS_SOLVE)
    assert m_out[0] == np.float32(m_hat)
    cdf, pdf = _truncated(stats.norm(scale=s_hat), m_hat)
    want, h = _grid_argmin(m_hat, cdf)
    assert abs(float(p[0]) - want) <= 2 * h + 1e-6 * m_hat
    # Eq.12 gives the minimum in terms of f(p*) alone; it equals Eq.6 only at a
    # root of Eq.11
    ps = float(p[0])
    eq12 = -ps * ps + m_hat * ps - m_hat * (m_hat - 2 * ps) ** 2 * pdf(ps)
    assert eq12 == pytest.approx(_eq6(ps, m_hat, cdf), rel=1e-5)
    assert 0 < ps < 0.5 * m_hat


@pytest.mark.parametrize("x", [3.0, 5.0, 8.0, 12.0])
@pytest.mark.parametrize("beta", [1.0, 0.02])
def test_laplacian_solver_minimises_eq6(x, beta):
    m = x * beta
    w = _group_with_moments(m, beta=beta)
    b_hat = float(np.mean(np.abs(w.astype(np.float64))))
    m_hat = float(np.abs(w).max())
    p, _ = R.select_analytic(w, R.LAPLACE_SOLVE)
    cdf, pdf = _truncated(stats.laplace(scale=b_hat), m_hat)
    want, h = _grid_argmin(m_hat, cdf)
    assert abs(float(p[0]) - want) <= 2 * h + 1e-6 * m_hat
    ps = float(p[0])
    eq12 = -ps * ps + m_hat * ps - m_hat * (m_hat - 2 * ps) ** 2 * pdf(ps)
    assert eq12 == pytest.approx(_eq6(ps, m_hat, cdf), rel=1e-5)


def test_logarithmic_fit_follows_the_gaussian_solver():
    # Section 5.1: ln(0.8614 x + 0.6079) approximates the optimal breakpoint of a
    # normalized Gaussian with range x (both in units of sigma).
    const = _constants()
    for x in np.linspace(2.5, 7.0, 10):
        w = _group_with_moments(float(x), sigma=1.0)
        fit, _ = R.select_analytic(w, R.GAUSS_FIT)
        solved, _ = R.select_analytic(w, R.GAUSS_SOLVE)
        s_hat = float(np.sqrt(np.mean(w.astype(np.float64) ** 2)))
        x_hat = float(np.abs(w).max()) / s_hat
        printed = s_hat * math.log(const["closed_form_slope"] * x_hat + const["closed_form_offset"])
        assert float(fit[0]) == pytest.approx(printed, rel=1e-6)
        assert abs(float(fit[0]) - float(solved[0])) < 0.012 * float(solved[0])


def test_selectors_scale_with_the_data():
    rng = np.random.default_rng(5)
    w = (rng.standard_normal((3, 5000)) * np.array([[0.01], [1.0], [30.0]])).astype(np.float32)
    for sel in (R.GAUSS_FIT, R.GAUSS_SOLVE, R.LAPLACE_SOLVE):
        p, m = R.select_analytic(w, sel)
        p8, m8 = R.select_analytic(w * np.float32(8.0), sel)
        np.testing.assert_allclose(p8, 8 * p, rtol=2e-7)
        np.testing.assert_array_equal(m8, 8 * m)
        pn, _ = R.select_analytic(-w, sel)
        np.testing.assert_array_equal(pn, p)
        assert ((p > 0) & (p < 0.5 * m)).all()
    # per-tensor = one flat channel
    p_t, m_t = R.select_analytic(w, R.GAUSS_SOLVE, mode=R.PER_TENSOR)
    p_f, m_f = R.select_analytic(w.reshape(1, -1), R.GAUSS_SOLVE)
    assert p_t.shape == (1,) and p_t[0] == p_f[0] and m_t[0] == m_f[0]


def test_selectors_on_degenerate_groups():
    w = np.zeros((3, 7), np.float32)
    w[1, 2] = np.nan
    w[2] = 0.5                                   # every magnitude equals m
    for sel in (R.GAUSS_FIT, R.GAUSS_SOLVE, R.LAPLACE_SOLVE):
        p, m = R.select_analytic(w, sel)
        assert p[0] == 0 and m[0] == 0
        assert np.isnan(p[1]) and np.isnan(m[1])
        assert 0 <= p[2] <= 0.25 + 1e-7 and m[2] == 0.5
    with pytest.raises(ValueError):
        R.select_analytic(w, 3)


def test_selected_breakpoints_are_near_the_empirical_optimum():
    # On samples that follow the assumed distribution, the error at the analytic
    # breakpoint is within a few percent of the exhaustive optimum of Eq.7.
    rng = np.random.default_rng(17)
    K = 400_000
    g = rng.standard_normal((1, K)).astype(np.float32)
    l = rng.laplace(0.0, 0.05, (1, K)).astype(np.float32)
    for w, sel in ((g, R.GAUSS_SOLVE), (g, R.GAUSS_FIT), (l, R.LAPLACE_SOLVE)):
        best = R.search(w, 4, 500)
        p, m = R.select_analytic(w, sel)
        got = R.mse(w, 4, p, m)
        assert got[0] >= best["mse"][0] * (1 - 1e-12)
        assert got[0] < 1.05 * best["mse"][0]


# ------------------------------------------------ error at a given breakpoint
def test_mse_matches_exact_rational_brute_force():
    bits, L = 3, 3
    m = Fraction(3 * 8, 64)
    p = Fraction(9, 64)                          # p/L and (m-p)/L are dyadic
    rng = np.random.default_rng(3)
    ints = rng.integers(-int(m * 256), int(m * 256) + 1, size=(4, 24))
    ints[:, 0] = int(m * 256)
    w = (ints / 256.0).astype(np.float32)
    got = R.mse(w, bits, np.full(4, float(p), np.float32), np.full(4, float(m), np.float32))
    for g in range(4):
        total = Fraction(0)
        for v in ints[g]:
            a = abs(Fraction(int(v), 256))
            levels = ([Fraction(j) * p / L for j in range(L + 1)] if a <= p
                      else [p + Fraction(j) * (m - p) / L for j in range(L + 1)])
            total += min((lv - a) ** 2 for lv in levels)
        assert got[g] == float(total / 24)


def test_mse_agrees_with_the_search_curve_and_the_quantizer():
    rng = np.random.default_rng(23)
    w = rng.laplace(0, 0.05, (6, 777)).astype(np.float32)
    out = R.search(w, 4, 50, want_curve=True)
    for k in (1, 17, 50):
        p = (out["m"] * np.float32(k / 50)).astype(np.float32)
        np.testing.assert_allclose(R.mse(w, 4, p, out["m"]) * 777, out["curve"][:, k - 1], rtol=1e-15)
    # off-grid breakpoint: the error of the dequantized weights, apart from the
    # end-point snap of the top codes (at most an ulp of p or m per element)
    p = (out["m"] * np.float32(0.3137)).astype(np.float32)
    _, _, w_hat = R.quantize(w, 4, p, out["m"])
    direct = ((w_hat.astype(np.float64) - w.astype(np.float64)) ** 2).mean(axis=1)
    np.testing.assert_allclose(R.mse(w, 4, p, out["m"]), direct, rtol=1e-5)
