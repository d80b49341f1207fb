"""ctypes binding of libmigration_step.so: one scheduling decision of Algorithm 1
(Section 6.3).  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmigration_step.so")
NONE, MIGRATE, INVALID_ARG, NO_PENDING = 0, 1, -1, -1
_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2605_06374_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        i32p, u8p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_uint8)
        L.migration_step_decide.restype = ctypes.c_int
        L.migration_step_decide.argtypes = [i32p, u8p, ctypes.c_int32, ctypes.c_int32, i32p, u8p,
                                            i32p, i32p, i32p]
        _lib = L
    return _lib


def migration_step_decide(progress, fail_stop, delta, next_pending, memory_feasible):
    """Returns (source, destination, micro_batch) or None; next_pending entries may be None."""
    i32p, u8p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_uint8)
    p = np.ascontiguousarray(progress, dtype=np.int32)
    f = np.ascontiguousarray([1 if x else 0 for x in fail_stop], dtype=np.uint8)
    nx = np.ascontiguousarray([NO_PENDING if x is None else int(x) for x in next_pending], dtype=np.int32)
    mem = np.ascontiguousarray([1 if x else 0 for x in memory_feasible], dtype=np.uint8)
    if not (len(p) == len(f) == len(nx) == len(mem)):
        raise ValueError("migration_step_decide: arrays differ in length")
    src, dst, mb = ctypes.c_int32(-1), ctypes.c_int32(-1), ctypes.c_int32(-1)
    rc = lib().migration_step_decide(p.ctypes.data_as(i32p), f.ctypes.data_as(u8p), len(p), int(delta),
                                     nx.ctypes.data_as(i32p), mem.ctypes.data_as(u8p),
                                     ctypes.byref(src), ctypes.byref(dst), ctypes.byref(mb))
    if rc < 0:
        raise ValueError(f"migration_step_decide: status {rc}")
    return (int(src.value), int(dst.value), int(mb.value)) if rc == MIGRATE else None
