"""ctypes binding of libpipeline_dag.so: iteration-time prediction of Section 5.2 (Eq. 2) over
the 1F1B and ZB-H1 chunk orders.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpipeline_dag.so")
OK, INVALID_ARG, BAD_SCHEDULE = 0, -1, -2
F, B, W = 0, 1, 2
_lib = None


class Chunk(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("microbatch", ctypes.c_int32)]


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2605_06374_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        cp, dp = ctypes.POINTER(Chunk), ctypes.POINTER(ctypes.c_double)
        for name in ("pipeline_dag_schedule_1f1b", "pipeline_dag_schedule_zbh1"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [ctypes.c_int32, ctypes.c_int32, cp]
        L.pipeline_dag_simulate.restype = ctypes.c_int
        L.pipeline_dag_simulate.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32, cp, dp,
                                            ctypes.c_double, dp, dp]
        _lib = L
    return _lib


def _schedule(fn, stages, microbatches, kinds):
    arr = (Chunk * (stages * kinds * microbatches))()
    rc = fn(int(stages), int(microbatches), arr)
    if rc != OK:
        raise ValueError(f"pipeline_dag schedule: status {rc}")
    per = kinds * microbatches
    return [[(arr[s * per + i].kind, arr[s * per + i].microbatch) for i in range(per)]
            for s in range(stages)]


def pipeline_dag_schedule_1f1b(stages, microbatches):
    return _schedule(lib().pipeline_dag_schedule_1f1b, stages, microbatches, 2)


def pipeline_dag_schedule_zbh1(stages, microbatches):
    return _schedule(lib().pipeline_dag_schedule_zbh1, stages, microbatches, 3)


def pipeline_dag_simulate(stages, microbatches, schedule, cost, p2p, want_starts=False):
    """schedule: per-stage lists of (kind, microbatch); cost: array [kinds][M][S]."""
    cost = np.ascontiguousarray(cost, dtype=np.float64)
    kinds = cost.shape[0]
    if cost.shape != (kinds, microbatches, stages):
        raise ValueError("cost must be [kinds][microbatches][stages]")
    flat = [c for order in schedule for c in order]
    if len(schedule) != stages or any(len(o) != kinds * microbatches for o in schedule):
        raise ValueError("schedule must hold kinds * microbatches chunks per stage")
    arr = (Chunk * len(flat))(*[Chunk(int(k), int(m)) for k, m in flat])
    total = ctypes.c_double(0.0)
    starts = np.zeros_like(cost) if want_starts else None
    rc = lib().pipeline_dag_simulate(
        int(stages), int(microbatches), int(kinds), arr,
        cost.ctypes.data_as(ctypes.POINTER(ctypes.c_double)), float(p2p), ctypes.byref(total),
        starts.ctypes.data_as(ctypes.POINTER(ctypes.c_double)) if want_starts else None)
    if rc != OK:
        raise ValueError(f"pipeline_dag_simulate: status {rc}")
    return (float(total.value), starts) if want_starts else float(total.value)
