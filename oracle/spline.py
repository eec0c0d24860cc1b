"""Oracle: natural cubic spline, written as the paper's four conditions.

TEST INFRASTRUCTURE ONLY - never imported by the product path.

Appendix "Cubic Spline Interpolation": on each interval [x_i, x_{i+1}] the
curve is S_i(x) = a_i + b_i (x-x_i) + c_i (x-x_i)^2 + d_i (x-x_i)^3, with
(2) interpolation at every knot, (3) continuous first and second derivatives
at interior knots, (4) zero second derivative at both ends.  The 4n unknowns
are found by solving those 4n linear equations directly.
"""
import numpy as np


def natural_spline_coeffs(x, y):
    """x strictly increasing, len >= 2.  Returns array [n, 4] of (a, b, c, d)."""
    x = np.asarray(x, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    n = len(x) - 1
    A = np.zeros((4 * n, 4 * n))
    rhs = np.zeros(4 * n)
    row = 0
    for i in range(n):
        h = x[i + 1] - x[i]
        # S_i(x_i) = y_i
        A[row, 4 * i] = 1.0
        rhs[row] = y[i]
        row += 1
        # S_i(x_{i+1}) = y_{i+1}
        A[row, 4 * i:4 * i + 4] = [1.0, h, h * h, h ** 3]
        rhs[row] = y[i + 1]
        row += 1
    for i in range(n - 1):
        h = x[i + 1] - x[i]
        # S_i'(x_{i+1}) = S_{i+1}'(x_{i+1})
        A[row, 4 * i + 1:4 * i + 4] = [1.0, 2 * h, 3 * h * h]
        A[row, 4 * (i + 1) + 1] = -1.0
        row += 1
        # S_i''(x_{i+1}) = S_{i+1}''(x_{i+1})
        A[row, 4 * i + 2:4 * i + 4] = [2.0, 6 * h]
        A[row, 4 * (i + 1) + 2] = -2.0
        row += 1
    # S_0''(x_0) = 0 ; S_{n-1}''(x_n) = 0
    A[row, 2] = 2.0
    row += 1
    hl = x[n] - x[n - 1]
    A[row, 4 * (n - 1) + 2:4 * (n - 1) + 4] = [2.0, 6 * hl]
    row += 1
    assert row == 4 * n
    return np.linalg.solve(A, rhs).reshape(n, 4)


def natural_spline_eval(x, coeffs, xq):
    """Evaluate at xq (inside [x_0, x_n])."""
    x = np.asarray(x, dtype=np.float64)
    xq = np.atleast_1d(np.asarray(xq, dtype=np.float64))
    i = np.clip(np.searchsorted(x, xq, side="right") - 1, 0, len(x) - 2)
    t = xq - x[i]
    a, b, c, d = coeffs[i].T
    return a + b * t + c * t * t + d * t ** 3
