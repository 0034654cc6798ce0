"""Soft-TopK operator ST_k of Sec. 3.2 / App. A, forward and backward, fp64, CPU.

TEST INFRASTRUCTURE, NOT PRODUCT.  The hot path uses the hard top-k; this
operator is kept because the paper states that it converges to the hard top-k
as the temperature goes to 0+, which gives a check of the oracle's top-k that
is not itself a sort-and-slice.

Definition (Sec. 3.2): ST_k(x)_i = f(x_i - lambda), f the Laplace CDF
f(z) = (1 + sgn(z)(1 - e^{-|z|})) / 2, with lambda chosen so the outputs sum
to k.  With x sorted in descending order and a split index m such that
x_m >= lambda >= x_{m+1}, App. A.1 reduces the constraint to the quadratic
S1 y^2 + 2 (k - m) y - S2 = 0 in y = e^lambda, S1 = sum_{i<=m} e^{-x_i},
S2 = sum_{i>m} e^{x_i}, whose positive root is Eq. (2).

The paper restricts m to 1..n-1.  The same quadratic degenerates cleanly at
the two ends (m = 0: y = S2 / 2k;  m = n: y = 2 (n - k) / S1) and both are
accepted here so that k = 1 reproduces the softmax whenever the largest
softmax probability is at most 1/2.

Everything is evaluated in log space (log S1, log S2) so that x / tau with a
tiny tau does not overflow.

Backward (App. A.2).  The threshold is defined implicitly by sum_i f(x_i - lambda) = k, so
    d lambda / d x_j = f'(x_j - lambda) / sum_i f'(x_i - lambda),
    d lambda / d k   = -1 / sum_i f'(x_i - lambda),          f'(z) = e^{-|z|} / 2,
and the outputs y_i = f(x_i / tau - lambda(x / tau, k)) follow by the chain rule.
``soft_topk_backward`` applies the transposed Jacobian to an upstream gradient g = dL/dy:
    dL/dx_j = (f'(z_j) / tau) (g_j - gbar),   dL/dk = gbar,   gbar = sum_i g_i w_i,
with z = x / tau - lambda and w_i = f'(z_i) / sum f'(z) the first of the two derivatives above.
The weights w are formed relative to the smallest |z| so that a cold temperature, where every
f'(z_i) underflows, still gives the finite ratios the formulas define.
"""
from __future__ import annotations

import math

import numpy as np


def laplace_cdf(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=np.float64)
    e = 0.5 * np.exp(-np.abs(z))
    return np.where(z >= 0, 1.0 - e, e)


def _log_sqrt_plus_abs(abs_d: float, log_e: float) -> float:
    """log( sqrt(d^2 + E) + |d| ) with E = exp(log_e), without overflow."""
    if log_e == -math.inf:
        return math.log(2.0 * abs_d) if abs_d > 0 else -math.inf
    half = 0.5 * log_e
    if abs_d == 0.0:
        return half
    log_d = math.log(abs_d)
    if half >= log_d:
        t = math.exp(log_d - half)
        return half + math.log(math.sqrt(t * t + 1.0) + t)
    t = math.exp(2.0 * (half - log_d))
    return log_d + math.log(math.sqrt(1.0 + t) + 1.0)


def _logsumexp(a: np.ndarray) -> float:
    if a.size == 0:
        return -math.inf
    m = float(a.max())
    return m + math.log(float(np.exp(a - m).sum()))


def soft_topk_lambda(x: np.ndarray, k: float):
    """Threshold lambda(x) of Eq. (2) and the split index m it was found at."""
    x = np.asarray(x, dtype=np.float64).reshape(-1)
    n = x.size
    if not 0.0 < k < n:
        raise ValueError("k must lie in the open interval (0, n)")
    xs = np.sort(x)[::-1]
    for m in range(0, n + 1):
        log_s1 = _logsumexp(-xs[:m])
        log_s2 = _logsumexp(xs[m:])
        d = k - m
        if m == 0:
            lam = log_s2 - math.log(2.0 * k)
        elif m == n:
            lam = math.log(2.0 * (n - k)) - log_s1
        elif d >= 0:
            # rationalised root: y = S2 / (sqrt(d^2 + S1 S2) + d)
            lam = log_s2 - _log_sqrt_plus_abs(d, log_s1 + log_s2)
        else:
            # y = (sqrt(d^2 + S1 S2) + |d|) / S1
            lam = _log_sqrt_plus_abs(-d, log_s1 + log_s2) - log_s1
        upper = xs[m - 1] if m >= 1 else math.inf
        lower = xs[m] if m < n else -math.inf
        if lower <= lam <= upper:
            return lam, m
    raise RuntimeError("no consistent split index")  # cannot happen: sum f is monotone in lambda


def soft_topk(x: np.ndarray, k: float, tau: float = 1.0) -> np.ndarray:
    """ST_k(x / tau): values in (0, 1) that sum to k, in the input's order."""
    x = np.asarray(x, dtype=np.float64)
    xt = x / tau
    lam, _ = soft_topk_lambda(xt, k)
    return laplace_cdf(xt - lam)


def laplace_pdf(z: np.ndarray) -> np.ndarray:
    """f'(z): the density of the Laplace distribution (App. A.2)."""
    return 0.5 * np.exp(-np.abs(np.asarray(z, dtype=np.float64)))


def threshold_weights(z: np.ndarray) -> np.ndarray:
    """w_j = f'(z_j) / sum_i f'(z_i) = d lambda / d x_j (App. A.2), without underflow of the sum."""
    a = np.abs(np.asarray(z, dtype=np.float64))
    e = np.exp(a.min() - a)
    return e / e.sum()


def soft_topk_backward(x: np.ndarray, k: float, tau: float, g: np.ndarray):
    """(dL/dx, dL/dk) of y = ST_k(x / tau) for the upstream gradient g = dL/dy (App. A.2)."""
    x = np.asarray(x, dtype=np.float64)
    g = np.asarray(g, dtype=np.float64)
    xt = x / tau
    lam, _ = soft_topk_lambda(xt, k)
    z = xt - lam
    gbar = float((g * threshold_weights(z)).sum())
    return laplace_pdf(z) * (g - gbar) / tau, gbar
