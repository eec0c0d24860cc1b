"""Pins for oracle/spline.py: the appendix's four conditions, exactness on
lines, and scipy's natural spline.  CPU only."""
import numpy as np
from scipy.interpolate import CubicSpline

from oracle.spline import natural_spline_coeffs, natural_spline_eval


def _data(seed, n):
    rng = np.random.default_rng(seed)
    x = np.cumsum(rng.integers(1, 5, n)).astype(float)
    return x, rng.standard_normal(n) * 3


def test_matches_scipy_natural():
    for seed, n in [(0, 2), (1, 3), (2, 6), (3, 11)]:
        x, y = _data(seed, n)
        c = natural_spline_coeffs(x, y)
        xq = np.linspace(x[0], x[-1], 101)
        ref = CubicSpline(x, y, bc_type="natural")(xq)
        np.testing.assert_allclose(natural_spline_eval(x, c, xq), ref, rtol=1e-10, atol=1e-12)


def test_conditions_hold():
    x, y = _data(4, 7)
    c = natural_spline_coeffs(x, y)
    h = np.diff(x)
    a, b, cc, d = c.T
    np.testing.assert_allclose(a, y[:-1], atol=1e-12)                                   # S_i(x_i) = y_i
    np.testing.assert_allclose(a + b * h + cc * h ** 2 + d * h ** 3, y[1:], atol=1e-11)  # S_i(x_{i+1}) = y_{i+1}
    np.testing.assert_allclose((b + 2 * cc * h + 3 * d * h ** 2)[:-1], b[1:], atol=1e-11)  # C1
    np.testing.assert_allclose((2 * cc + 6 * d * h)[:-1], 2 * cc[1:], atol=1e-11)        # C2
    assert abs(cc[0]) < 1e-12 and abs(2 * cc[-1] + 6 * d[-1] * h[-1]) < 1e-11            # natural ends


def test_reproduces_a_line():
    x = np.array([1.0, 2, 4, 8, 11])
    y = 3.0 - 0.5 * x
    c = natural_spline_coeffs(x, y)
    xq = np.arange(1, 12, dtype=float)
    np.testing.assert_allclose(natural_spline_eval(x, c, xq), 3.0 - 0.5 * xq, atol=1e-12)


def test_known_three_point_spline():
    # knots (0,0),(1,1),(2,0): by symmetry S''(1) = -3, S(0.5) = 11/16
    x = np.array([0.0, 1, 2])
    y = np.array([0.0, 1, 0])
    c = natural_spline_coeffs(x, y)
    assert abs(natural_spline_eval(x, c, 0.5)[0] - 11.0 / 16.0) < 1e-13
    assert abs(2 * c[1, 2] + 3.0) < 1e-12
