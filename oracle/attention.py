"""ctypes front end of the C fp64 oracle (oracle/varlen_attn_oracle.c).

Test infrastructure: document-masked causal attention and its gradients evaluated from the
plain definition (Section 5.2: packed documents, block-diagonal mask; decoder-only models,
hence causal).  Inputs are numpy arrays (any float dtype; converted exactly to float64).
Shapes: q, d_o [N, Hq, d]; k, v [N, Hkv, d]; cu_seqlens int32 [B+1].
Returns float64 arrays: o [N, Hq, d], lse [Hq, N], dq [N, Hq, d], dk, dv [N, Hkv, d].
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional, Tuple

import numpy as np

from . import build as _build

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build(force=True)
        _lib = ctypes.CDLL(path)
        _lib.vao_set_threads.restype = ctypes.c_int
        _lib.vao_set_threads.argtypes = [ctypes.c_int]
        for name in ("vao_fwd_rows", "vao_dq_rows", "vao_dkv_rows", "vao_fwd", "vao_bwd"):
            getattr(_lib, name).restype = ctypes.c_int
    return _lib


def set_threads(n: int = 0) -> int:
    """Set (n > 0) or query (n == 0) the OpenMP thread count the oracle uses."""
    return int(_load().vao_set_threads(int(n)))


def _f64(x) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(x), dtype=np.float64)


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _dims(q, k, cu):
    n, hq, d = q.shape
    n2, hkv, d2 = k.shape
    assert n == n2 and d == d2 and hq % hkv == 0
    cu = np.ascontiguousarray(cu, dtype=np.int32)
    assert cu.ndim == 1 and cu.size >= 2
    return n, cu.size - 1, hq, hkv, d, cu


def _scalars(n, b, hq, hkv, d, scale):
    return (ctypes.c_int32(n), ctypes.c_int32(b), ctypes.c_int32(hq), ctypes.c_int32(hkv),
            ctypes.c_int32(d), ctypes.c_double(scale))


def _check(rc, what):
    if rc != 0:
        raise ValueError(f"oracle {what} failed with code {rc} (bad cu_seqlens or heads)")


def fwd(q, k, v, cu_seqlens, scale, rows=None) -> Tuple[np.ndarray, np.ndarray]:
    """O and LSE for all tokens, or for the listed token indices only
    (then o is [len(rows), Hq, d] and lse is [Hq, len(rows)])."""
    q, k, v = _f64(q), _f64(k), _f64(v)
    n, b, hq, hkv, d, cu = _dims(q, k, cu_seqlens)
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        assert rows.size == 0 or (rows.min() >= 0 and rows.max() < n)
    nr = n if rows is None else int(rows.size)
    o = np.zeros((nr, hq, d), dtype=np.float64)
    lse = np.zeros((hq, nr), dtype=np.float64)
    rc = _load().vao_fwd_rows(*_scalars(n, b, hq, hkv, d, scale), _ptr(q), _ptr(k), _ptr(v),
                              _ptr(cu), _ptr(rows), ctypes.c_int32(nr), _ptr(o), _ptr(lse))
    _check(rc, "fwd")
    return o, lse


def dq_rows(q, k, v, d_o, cu_seqlens, scale, rows=None) -> Tuple[np.ndarray, np.ndarray]:
    """dQ [len(rows), Hq, d] and D = rowsum(dO * O) [Hq, len(rows)] (rows None: all)."""
    q, k, v, d_o = _f64(q), _f64(k), _f64(v), _f64(d_o)
    n, b, hq, hkv, d, cu = _dims(q, k, cu_seqlens)
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        assert rows.size == 0 or (rows.min() >= 0 and rows.max() < n)
    nr = n if rows is None else int(rows.size)
    dq = np.zeros((nr, hq, d), dtype=np.float64)
    dd = np.zeros((hq, nr), dtype=np.float64)
    rc = _load().vao_dq_rows(*_scalars(n, b, hq, hkv, d, scale), _ptr(q), _ptr(k), _ptr(v),
                             _ptr(d_o), _ptr(cu), _ptr(rows), ctypes.c_int32(nr), _ptr(dq),
                             _ptr(dd))
    _check(rc, "dq_rows")
    return dq, dd


def dkv_rows(q, k, v, d_o, lse, dsum, cu_seqlens, scale, rows=None):
    """dK, dV [len(rows), Hkv, d] for the listed key tokens, given full LSE and D [Hq, N]."""
    q, k, v, d_o = _f64(q), _f64(k), _f64(v), _f64(d_o)
    lse, dsum = _f64(lse), _f64(dsum)
    n, b, hq, hkv, d, cu = _dims(q, k, cu_seqlens)
    assert lse.shape == (hq, n) and dsum.shape == (hq, n)
    if rows is not None:
        rows = np.ascontiguousarray(rows, dtype=np.int32)
        assert rows.size == 0 or (rows.min() >= 0 and rows.max() < n)
    nr = n if rows is None else int(rows.size)
    dk = np.zeros((nr, hkv, d), dtype=np.float64)
    dv = np.zeros((nr, hkv, d), dtype=np.float64)
    rc = _load().vao_dkv_rows(*_scalars(n, b, hq, hkv, d, scale), _ptr(q), _ptr(k), _ptr(v),
                              _ptr(d_o), _ptr(lse), _ptr(dsum), _ptr(cu), _ptr(rows),
                              ctypes.c_int32(nr), _ptr(dk), _ptr(dv))
    _check(rc, "dkv_rows")
    return dk, dv


def bwd(q, k, v, d_o, cu_seqlens, scale):
    """dQ, dK, dV for the whole microbatch (the forward is recomputed inside)."""
    q, k, v, d_o = _f64(q), _f64(k), _f64(v), _f64(d_o)
    n, b, hq, hkv, d, cu = _dims(q, k, cu_seqlens)
    dq = np.zeros((n, hq, d), dtype=np.float64)
    dk = np.zeros((n, hkv, d), dtype=np.float64)
    dv = np.zeros((n, hkv, d), dtype=np.float64)
    rc = _load().vao_bwd(*_scalars(n, b, hq, hkv, d, scale), _ptr(q), _ptr(k), _ptr(v),
                         _ptr(d_o), _ptr(cu), _ptr(dq), _ptr(dk), _ptr(dv))
    _check(rc, "bwd")
    return dq, dk, dv
