"""ctypes binding of libtp_select.so: TP subgroup selection of Section 6.1 (Eq. 3, Eq. 4).
Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libtp_select.so")
OK, INVALID_ARG, NO_FEASIBLE_DEGREE = 0, -1, 1
ROLE_FAIL_STOP, ROLE_MEMBER, ROLE_STANDBY = 0, 1, 2
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2605_06374_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        L.tp_select_subgroup.restype = ctypes.c_int
        L.tp_select_subgroup.argtypes = [ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_uint8),
                                         ctypes.c_int32, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32),
                                         ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int32)]
        _lib = L
    return _lib


def tp_select_subgroup(throughput, fail_stop, k_min):
    """throughput: p_i per device of G; fail_stop: indices in F_stop.  Returns (degree,
    members, standby, aggregate throughput); degree 0 when no feasible degree exists."""
    p = np.ascontiguousarray(throughput, dtype=np.float64)
    n = len(p)
    flags = np.zeros(n, dtype=np.uint8)
    flags[list(fail_stop)] = 1
    role = np.zeros(n, dtype=np.int32)
    degree, agg = ctypes.c_int32(0), ctypes.c_double(0.0)
    rc = lib().tp_select_subgroup(p.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                  flags.ctypes.data_as(ctypes.POINTER(ctypes.c_uint8)), n, int(k_min),
                                  ctypes.byref(degree), ctypes.byref(agg),
                                  role.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)))
    if rc < 0:
        raise ValueError(f"tp_select_subgroup: status {rc}")
    members = [i for i in range(n) if role[i] == ROLE_MEMBER]
    standby = [i for i in range(n) if role[i] == ROLE_STANDBY]
    return int(degree.value), members, standby, float(agg.value)
