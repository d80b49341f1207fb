"""Pins of the micro-batch time oracle (Section 5.2, Eq. 1 and the 25 % rule) against what the
mathematics and the paper fix, none of them a re-call of the oracle's own routine."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import mb_time as O


def test_tokens_and_sum_sq_by_hand():
    assert O.tokens_and_sum_sq([0, 3, 3, 10]) == (10, 9 + 0 + 49)
    assert O.tokens_and_sum_sq([0, 4096]) == (4096, 4096 * 4096)
    with pytest.raises(ValueError):
        O.tokens_and_sum_sq([0, 5, 4])
    with pytest.raises(ValueError):
        O.tokens_and_sum_sq([1, 5])


def test_quadratic_term_of_one_4k_document_is_four_times_four_1k_documents():
    """Section 2.2: a 4K-token sequence costs about four times four packed 1K sequences in
    attention; with Eq. 1 the quadratic terms are in the ratio sum l^2 = 4 exactly."""
    n1, s1 = O.tokens_and_sum_sq([0, 4096])
    n4, s4 = O.tokens_and_sum_sq([0, 1024, 2048, 3072, 4096])
    assert n1 == n4 == 4096 and s1 == 4 * s4
    alpha, beta = 0.0, 7.5e-6
    assert O.predict(alpha, beta, n1, s1) == 4 * O.predict(alpha, beta, n4, s4)


def test_fit_recovers_planted_coefficients_exactly_representable():
    rng = np.random.default_rng(7)
    n = np.full(40, 4096)
    s = rng.integers(200_000, 16_777_216, size=40)
    alpha, beta = 0.015625, 2.0 ** -17          # products below are exact in fp64
    t = alpha * n + beta * s
    a, b = O.fit(n, s, t)
    assert abs(a - alpha) <= 1e-12 * alpha and abs(b - beta) <= 1e-12 * beta


def test_two_points_match_cramers_rule_in_rationals():
    n, s, t = [4096, 8192], [2_000_000, 30_000_000], [Fraction(131, 10), Fraction(977, 10)]
    det = Fraction(n[0] * s[1] - n[1] * s[0])
    alpha = (t[0] * s[1] - t[1] * s[0]) / det
    beta = (n[0] * t[1] - n[1] * t[0]) / det
    a, b = O.fit(n, s, [float(x) for x in t])
    assert abs(a - float(alpha)) <= 1e-10 * abs(float(alpha))
    assert abs(b - float(beta)) <= 1e-10 * abs(float(beta))


def test_residual_is_orthogonal_to_both_regressors():
    rng = np.random.default_rng(11)
    n = rng.integers(2048, 8193, size=64).astype(np.float64)
    s = np.array([int(x) ** 2 // rng.integers(1, 30) for x in n], dtype=np.float64)
    t = 3e-3 * n + 9e-7 * s + rng.normal(0, 0.5, size=64)
    a, b = O.fit(n, s, t)
    r = t - (a * n + b * s)
    assert abs(r @ n) <= 1e-8 * np.linalg.norm(t) * np.linalg.norm(n)
    assert abs(r @ s) <= 1e-8 * np.linalg.norm(t) * np.linalg.norm(s)


def test_unidentifiable_profiles_are_refused():
    with pytest.raises(ValueError):
        O.fit([4096], [1000], [1.0])
    with pytest.raises(ValueError):
        O.fit([4096, 4096, 4096], [5000, 5000, 5000], [1.0, 1.1, 0.9])   # identical rows
    with pytest.raises(ValueError):
        O.fit([100, 200], [1000, 2000], [1.0, 2.0])                      # collinear columns


def test_twenty_five_percent_rule_boundary():
    assert not O.is_suspicious(125.0, 100.0)          # exactly 25 % above: benign
    assert O.is_suspicious(125.0000001, 100.0)
    assert not O.is_suspicious(90.0, 100.0)
    assert O.is_suspicious(111.0, 100.0, threshold=0.1)


def test_mape_by_hand():
    # predictions 10 and 20 against observations 8 and 25: (2/8 + 5/25) / 2 = 22.5 %
    assert abs(O.mape_percent(1.0, 0.0, [10, 20], [0, 0], [8.0, 25.0]) - 22.5) < 1e-12
