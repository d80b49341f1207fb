"""Oracle (test infrastructure, CPU, fp64): micro-batch time model of Section 5.2.

Eq. 1 models the execution time of a packed micro-batch with documents l_1..l_k (sum N) as
T_MB ~ alpha * N + beta * sum_i l_i^2, alpha and beta being profiled in a warm-up phase; the
Detector treats a change point as fail-slow only if the observed time exceeds the predicted
healthy time by more than 25 % (end of Section 5.2).  Plain definitions, written out:
ordinary least squares through numpy's lstsq, the prediction as the formula, the filter as
the inequality.  Only tests, smoke() and bench.py's baseline leg may import this module.

Pins: tests/test_oracle_pins_mb_time.py (exact recovery of planted coefficients, the 2x2 case
solved in rational arithmetic, the normal equations as an invariant, the 4K-vs-4x1K ratio of
Section 2.2, the boundary of the 25 % rule).
"""
from __future__ import annotations

import numpy as np


def tokens_and_sum_sq(cu_seqlens):
    """N = sum l_i and sum l_i^2 of a packed micro-batch, exact Python integers."""
    cu = [int(x) for x in cu_seqlens]
    if len(cu) < 2 or cu[0] != 0 or any(b < a for a, b in zip(cu, cu[1:])):
        raise ValueError("malformed cu_seqlens")
    lengths = [b - a for a, b in zip(cu, cu[1:])]
    return sum(lengths), sum(l * l for l in lengths)


def fit(n_tokens, sum_sq, times):
    """Least-squares alpha, beta of Eq. 1 (no intercept) over the profiled micro-batches."""
    x = np.stack([np.asarray(n_tokens, dtype=np.float64), np.asarray(sum_sq, dtype=np.float64)], axis=1)
    t = np.asarray(times, dtype=np.float64)
    if x.shape[0] < 2 or x.shape[0] != t.shape[0]:
        raise ValueError("need at least two profiled micro-batches")
    scale = np.sqrt((x * x).mean(axis=0))           # columns differ by ~1e4: solve scaled
    if not np.all(scale > 0):
        raise ValueError("degenerate profile")
    theta, _res, rank, _sv = np.linalg.lstsq(x / scale, t, rcond=1e-12)
    if rank < 2:
        raise ValueError("alpha and beta are not identifiable from this profile")
    alpha, beta = theta / scale
    return float(alpha), float(beta)


def predict(alpha, beta, n_tokens, sum_sq):
    """Eq. 1."""
    return alpha * float(n_tokens) + beta * float(sum_sq)


def mape_percent(alpha, beta, n_tokens, sum_sq, times):
    t = np.asarray(times, dtype=np.float64)
    p = np.array([predict(alpha, beta, n, s) for n, s in zip(n_tokens, sum_sq)])
    return float(np.mean(np.abs(p - t) / t) * 100.0)


def is_suspicious(observed, predicted, threshold=0.25):
    """True iff the observed time exceeds the predicted healthy time by more than the
    threshold (25 % in the paper): such a change point goes on to validation."""
    return observed > predicted * (1.0 + threshold)
