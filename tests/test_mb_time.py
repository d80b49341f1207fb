"""Micro-batch time predictor (host library) against the oracle, on seeded profiles shaped like
the length-skew sweep (fixed N = 4096, document-length medians 32 .. 4096), and its error paths."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import mb_time as O
from paper_2605_06374_amd import mb_time as M
from paper_2605_06374_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "mb_time.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(mb_time_[a-z_]+)\s*\(", text)))
    assert {"mb_time_features", "mb_time_fit", "mb_time_predict", "mb_time_mape_percent",
            "mb_time_is_suspicious"} <= set(names)
    lib = ctypes.CDLL(M.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert ctypes.sizeof(M.Model) == 16


def sweep_profile(noise, seed, vary_n=False):
    rng = np.random.default_rng(seed)
    feats = [O.tokens_and_sum_sq(W.config(5, microbatch=i).cu_seqlens) for i in range(64)]
    n = np.array([f[0] for f in feats], dtype=np.int64)
    s = np.array([f[1] for f in feats], dtype=np.int64)
    if vary_n:                                       # two micro-batches of the kind, packed together
        n[::2] *= 2
        s[::2] *= 2
    t = 0.0185 * n + 6.3e-6 * s                      # microseconds, like the measured sweep
    return n, s, t * (1.0 + noise * rng.standard_normal(64))


def test_features_bit_exact_on_all_configs():
    for k in (1, 2, 3, 4):
        cu = W.config(k).cu_seqlens
        assert M.mb_time_features(cu) == O.tokens_and_sum_sq(cu)
    for i in range(64):
        cu = W.config(5, microbatch=i).cu_seqlens
        assert M.mb_time_features(cu) == O.tokens_and_sum_sq(cu)
    assert M.mb_time_features([0, 0, 7, 7]) == (7, 49)            # empty documents
    assert M.mb_time_features([0, 2 ** 31 - 1]) == (2 ** 31 - 1, (2 ** 31 - 1) ** 2)   # int64 range


@pytest.mark.parametrize("noise,seed", [(0.0, 1), (0.03, 2), (0.2, 3)])
def test_fit_predict_mape_match_oracle(noise, seed):
    n, s, t = sweep_profile(noise, seed, vary_n=True)
    a, b = O.fit(n, s, t)
    m = M.mb_time_fit(n, s, t)
    assert abs(m.alpha - a) <= 1e-9 * abs(a) and abs(m.beta - b) <= 1e-9 * abs(b)
    for i in (0, 7, 63):
        want = O.predict(a, b, int(n[i]), int(s[i]))
        assert abs(M.mb_time_predict(m, int(n[i]), int(s[i])) - want) <= 1e-9 * abs(want)
    assert abs(M.mb_time_mape_percent(m, n, s, t) - O.mape_percent(a, b, n, s, t)) <= 1e-7
    if noise == 0.0:
        assert M.mb_time_mape_percent(m, n, s, t) < 1e-9


def test_filter_matches_oracle_around_the_threshold():
    for obs, pred, thr in ((125.0, 100.0, 0.25), (125.0000001, 100.0, 0.25), (80.0, 100.0, 0.25),
                           (111.0, 100.0, 0.1), (3.75e-3, 3e-3, 0.25), (3.7500001e-3, 3e-3, 0.25)):
        assert M.mb_time_is_suspicious(obs, pred, thr) == O.is_suspicious(obs, pred, thr)


def test_error_paths():
    with pytest.raises(ValueError):
        M.mb_time_features([0, 5, 4])
    with pytest.raises(ValueError):
        M.mb_time_features([1, 5])
    with pytest.raises(ValueError):
        M.mb_time_fit([4096], [1000], [1.0])                              # one sample
    with pytest.raises(ValueError):
        M.mb_time_fit([4096] * 3, [5000] * 3, [1.0, 1.1, 0.9])            # identical rows
    with pytest.raises(ValueError):
        M.mb_time_fit([100, 200], [1000, 2000], [1.0, 2.0])               # collinear columns
    with pytest.raises(ValueError):
        M.mb_time_fit([100, 200], [1000, 5000], [1.0, float("nan")])
    lib = M.lib()
    assert lib.mb_time_fit(None, None, None, 3, None) == M.INVALID_ARG
    assert np.isnan(lib.mb_time_mape_percent(None, None, None, None, 0))


def test_fixed_n_profile_is_identifiable_like_the_sweep():
    """With N fixed (the paper's setting) alpha * N acts as the constant term."""
    n, s, t = sweep_profile(0.0, 4)
    m = M.mb_time_fit(n, s, t)
    assert abs(m.alpha - 0.0185) <= 1e-9 and abs(m.beta - 6.3e-6) <= 1e-15
