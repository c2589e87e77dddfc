"""Oracle of the batch-duration model (test infrastructure, not product code).

Sec. 4.2 "Relationship Between the Number of Tokens and the Batch Duration", Eq. 9: the duration
of a prefill batch is modelled as a line in its uncached tokens utok(p), the duration of a decode
batch as a line in its request count req(d); slope and intercept come from a linear fit of
measured points.  The paper does not name the fit; the reading taken here is ordinary least
squares, and the strength of a linear relationship (the paper's comparison of total against
uncached tokens) is reported as the coefficient of determination.

Everything is the textbook definition written out in fp64 with numpy.  Only tests import this.
"""
from __future__ import annotations

import numpy as np


def fit_line(units, seconds):
    """(alpha, beta) minimising sum_i (seconds_i - alpha * units_i - beta)^2  (Eq. 9's slope and intercept)."""
    u = np.asarray(units, np.float64)
    s = np.asarray(seconds, np.float64)
    if u.ndim != 1 or u.shape != s.shape or len(u) < 2:
        raise ValueError("need two equally long vectors of at least two points")
    du = u - u.mean()
    sxx = float(np.sum(du * du))
    if sxx == 0.0:
        raise ValueError("all points have the same abscissa")
    alpha = float(np.sum(du * (s - s.mean()))) / sxx
    beta = float(s.mean()) - alpha * float(u.mean())
    return alpha, beta


def predict(alpha, beta, units):
    """Eq. 9: L(batch) = alpha * units + beta."""
    return alpha * np.asarray(units, np.float64) + beta


def r_squared(units, seconds, alpha, beta):
    """1 - (sum of squared residuals) / (sum of squared deviations of the durations from their mean)."""
    s = np.asarray(seconds, np.float64)
    res = s - predict(alpha, beta, units)
    tot = float(np.sum((s - s.mean()) ** 2))
    if tot == 0.0:
        return 1.0 if float(np.sum(res * res)) == 0.0 else 0.0
    return 1.0 - float(np.sum(res * res)) / tot


def mean_abs_rel_error(units, seconds, alpha, beta):
    s = np.asarray(seconds, np.float64)
    return float(np.mean(np.abs(predict(alpha, beta, units) - s) / s))
