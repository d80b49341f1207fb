"""ctypes binding of libmb_time.so: the micro-batch time predictor of Section 5.2 (Eq. 1) and
the 25 % filter.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmb_time.so")
OK, INVALID_ARG, BAD_CU_SEQLENS, NOT_IDENTIFIABLE = 0, -1, -2, -3
_lib = None


class Model(ctypes.Structure):
    _fields_ = [("alpha", ctypes.c_double), ("beta", ctypes.c_double)]


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2605_06374_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        i64p, dp, mp = ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_double), ctypes.POINTER(Model)
        L.mb_time_features.restype = ctypes.c_int
        L.mb_time_features.argtypes = [ctypes.POINTER(ctypes.c_int32), ctypes.c_int32, i64p, i64p]
        L.mb_time_fit.restype = ctypes.c_int
        L.mb_time_fit.argtypes = [i64p, i64p, dp, ctypes.c_int32, mp]
        L.mb_time_predict.restype = ctypes.c_double
        L.mb_time_predict.argtypes = [mp, ctypes.c_int64, ctypes.c_int64]
        L.mb_time_mape_percent.restype = ctypes.c_double
        L.mb_time_mape_percent.argtypes = [mp, i64p, i64p, dp, ctypes.c_int32]
        L.mb_time_is_suspicious.restype = ctypes.c_int
        L.mb_time_is_suspicious.argtypes = [ctypes.c_double, ctypes.c_double, ctypes.c_double]
        _lib = L
    return _lib


def _i64(x):
    a = np.ascontiguousarray(x, dtype=np.int64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64))


def _f64(x):
    a = np.ascontiguousarray(x, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def mb_time_features(cu_seqlens):
    cu = np.ascontiguousarray(cu_seqlens, dtype=np.int32)
    n, s = ctypes.c_int64(0), ctypes.c_int64(0)
    rc = lib().mb_time_features(cu.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)),
                                len(cu) - 1, ctypes.byref(n), ctypes.byref(s))
    if rc != OK:
        raise ValueError(f"mb_time_features: status {rc}")
    return int(n.value), int(s.value)


def mb_time_fit(n_tokens, sum_sq, times) -> Model:
    (na, npz), (sa, sp), (ta, tp) = _i64(n_tokens), _i64(sum_sq), _f64(times)
    if not (len(na) == len(sa) == len(ta)):
        raise ValueError("mb_time_fit: arrays differ in length")
    m = Model()
    rc = lib().mb_time_fit(npz, sp, tp, len(ta), ctypes.byref(m))
    if rc != OK:
        raise ValueError(f"mb_time_fit: status {rc}")
    return m


def mb_time_predict(model: Model, n_tokens: int, sum_sq: int) -> float:
    return float(lib().mb_time_predict(ctypes.byref(model), int(n_tokens), int(sum_sq)))


def mb_time_mape_percent(model: Model, n_tokens, sum_sq, times) -> float:
    (na, npz), (sa, sp), (ta, tp) = _i64(n_tokens), _i64(sum_sq), _f64(times)
    return float(lib().mb_time_mape_percent(ctypes.byref(model), npz, sp, tp, len(ta)))


def mb_time_is_suspicious(observed: float, predicted: float, threshold: float = 0.25) -> bool:
    return bool(lib().mb_time_is_suspicious(float(observed), float(predicted), float(threshold)))
