"""Shared test utilities: oracle evaluation of a workload (full or on sampled rows) and the
error metrics.  Expected values always come from oracle/, never from the HIP path."""
from __future__ import annotations

import numpy as np

from oracle import attention as oracle
from oracle import plan as oplan
from paper_2605_06374_amd import workloads as W

TOL_O = 1e-2      # max |x - y| / max |y|, forward output
TOL_GRAD = 2e-2   # same, dQ / dK / dV
TOL_LSE = 1e-3    # |x - y| <= TOL_LSE * max(1, |y|)
# Row-wise gate (catches a misplaced, missing or stale row that the tensor-scale gate could
# miss): max_i |x_i - y_i| over the d-vector of a (token, head) <= TOL_ROW * max(max_i |y_i| of
# that vector, rms of the tensor).  The error of a row follows the magnitude of the terms summed
# into it, not of the result (a row whose terms cancel is small, its rounding error is not),
# hence the floor at the tensor's rms.  O: 2.5 times the tensor-scale tolerance.  Gradients: the
# backward reads O as the forward stored it (bf16), so D = rowsum(dO * O) carries 2^-9 of
# sum |dO O|, which enters dS = P (dP - D) of the first rows of a document (few keys, P not small,
# dP - D small) at up to a tenth of their size; measured worst rows 1e-2 .. 6e-2.
TOL_ROW_O = 2.5e-2
TOL_ROW_GRAD = 0.15


def f64_values(w, values=None):
    vals = values if values is not None else w.values()
    return {n: W.bf16_bits_to_f32(b).astype(np.float64) for n, b in vals.items()}


def e1(x, y):
    """Tensor-scale relative error: max |x - y| / max |y|."""
    den = np.abs(y).max()
    return float(np.abs(x - y).max() / den) if den > 0 else float(np.abs(x - y).max())


def e2(x, y):
    """Element-wise error relative to max(|y_i|, rms of the element's d-vector)."""
    rms = np.sqrt((y * y).mean(axis=-1, keepdims=True))
    den = np.maximum(np.abs(y), rms)
    den = np.where(den > 0, den, 1.0)
    return float((np.abs(x - y) / den).max())


def e_row(x, y):
    """Row-wise error: max |x - y| over a d-vector relative to max(max |y| of it, tensor rms)."""
    rms = float(np.sqrt((y * y).mean()))
    den = np.maximum(np.abs(y).max(axis=-1), rms)
    den = np.where(den > 0, den, 1.0)
    return float((np.abs(x - y).max(axis=-1) / den).max())


def oracle_full(w, values=None):
    v = f64_values(w, values)
    cu, s = w.cu_seqlens, w.softmax_scale
    o, lse = oracle.fwd(v["q"], v["k"], v["v"], cu, s)
    dq, dk, dv = oracle.bwd(v["q"], v["k"], v["v"], v["do"], cu, s)
    return {"o": o, "lse": lse, "dq": dq, "dk": dk, "dv": dv}


def assert_close_full(got, ref, label="", row_tol_scale=1.0):
    errs = {}
    for name, tol in (("o", TOL_O), ("dq", TOL_GRAD), ("dk", TOL_GRAD), ("dv", TOL_GRAD)):
        assert np.isfinite(got[name]).all(), f"{label} {name}: non-finite output"
        errs[name] = (e1(got[name], ref[name]), e_row(got[name], ref[name]))
        assert errs[name][0] <= tol, f"{label} {name}: E1 {errs[name][0]:.3e} > {tol}"
        tol2 = (TOL_ROW_O if name == "o" else TOL_ROW_GRAD) * row_tol_scale
        assert errs[name][1] <= tol2, f"{label} {name}: row-wise {errs[name][1]:.3e} > {tol2}"
    dl = np.abs(got["lse"] - ref["lse"]) / np.maximum(1.0, np.abs(ref["lse"]))
    assert dl.max() <= TOL_LSE, f"{label} lse: {dl.max():.3e}"
    errs["lse"] = (float(dl.max()), float(dl.max()))
    return errs


def interesting_rows(cu, n_random, rng, tile=128):
    """Document edges, tile edges inside documents, and random tokens."""
    cu = [int(x) for x in cu]
    rows = set()
    for b in range(len(cu) - 1):
        s, e = cu[b], cu[b + 1]
        if e == s:
            continue
        for t in (s, s + 1, e - 1, e - 2, s + tile - 1, s + tile, e - 1 - (e - 1 - s) % tile):
            if s <= t < e:
                rows.add(t)
    n = cu[-1]
    rows.update(int(x) for x in rng.integers(0, n, size=n_random))
    return np.array(sorted(rows), dtype=np.int32)


def key_rows_cheap(cu, n_random, rng, window=48, short=1536):
    """Key tokens whose dK/dV the oracle can evaluate cheaply: anywhere in documents up to
    `short` tokens, and within the last `window` tokens of longer ones."""
    cu = [int(x) for x in cu]
    cand = []
    for b in range(len(cu) - 1):
        s, e = cu[b], cu[b + 1]
        if e == s:
            continue
        lo = s if e - s <= short else e - window
        cand.append((lo, e))
    keys = set()
    for lo, e in cand:
        keys.add(e - 1)
        keys.add(lo)
    for _ in range(n_random):
        lo, e = cand[int(rng.integers(0, len(cand)))]
        keys.add(int(rng.integers(lo, e)))
    return np.array(sorted(keys), dtype=np.int32)


def oracle_rows(w, rows, values=None):
    v = f64_values(w, values)
    cu, s = w.cu_seqlens, w.softmax_scale
    o, lse = oracle.fwd(v["q"], v["k"], v["v"], cu, s, rows=rows)
    dq, _ = oracle.dq_rows(v["q"], v["k"], v["v"], v["do"], cu, s, rows=rows)
    return {"o": o, "lse": lse, "dq": dq}


def oracle_keys(w, keys, values=None):
    """dK, dV for the listed key tokens; LSE and D are evaluated (by the oracle) only for the
    query rows those keys can see, everything else stays NaN so that any use shows."""
    v = f64_values(w, values)
    cu, s = w.cu_seqlens, w.softmax_scale
    doc = None
    cu_l = [int(x) for x in cu]
    need = set()
    for j in keys:
        b = max(i for i in range(len(cu_l) - 1) if cu_l[i] <= j < cu_l[i + 1])
        need.update(range(int(j), cu_l[b + 1]))
    need = np.array(sorted(need), dtype=np.int32)
    _, lse_r = oracle.fwd(v["q"], v["k"], v["v"], cu, s, rows=need)
    _, d_r = oracle.dq_rows(v["q"], v["k"], v["v"], v["do"], cu, s, rows=need)
    lse = np.full((w.n_q_heads, w.n_tokens), np.nan)
    dsum = np.full((w.n_q_heads, w.n_tokens), np.nan)
    lse[:, need] = lse_r
    dsum[:, need] = d_r
    dk, dv = oracle.dkv_rows(v["q"], v["k"], v["v"], v["do"], lse, dsum, cu, s, rows=keys)
    assert np.isfinite(dk).all() and np.isfinite(dv).all()
    return {"dk": dk, "dv": dv}
