"""ctypes binding of libmigration_plan.so: the loop of Algorithm 1 (Section 6.3) around a
slot-by-slot pipeline simulation.  Argument marshalling only."""
from __future__ import annotations

import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libmigration_plan.so")
OK, INVALID_ARG, UNSCHEDULABLE, MOVES_OVERFLOW = 0, -1, -2, -3
_lib = None


class Move(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("slot", "stage", "source", "destination", "group",
                                              "micro_batch")]


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2605_06374_amd.build`")
        L = ctypes.CDLL(LIB_PATH)
        i32, i32p, u8p = ctypes.c_int32, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_uint8)
        L.migration_plan_run.restype = ctypes.c_int
        L.migration_plan_run.argtypes = [i32, i32, i32, i32p, i32p, u8p, i32p, i32, i32, i32, i32p,
                                         i32p, i32p, ctypes.POINTER(Move), i32, i32p, i32p]
        _lib = L
    return _lib


def migration_plan_run(n_groups, n_stages, n_micro, f_cost, b_cost, fail_stop, capacity, delta,
                       p2p=0, migrate=True, assignment=None, moves_capacity=None):
    """Returns a dict with iteration_time, makespan [group], executed [group, micro, stage] and
    migrations [(slot, stage, source, destination, (group, micro_batch))].  Raises ValueError on
    invalid arguments, RuntimeError when the workloads cannot all run."""
    i32p, u8p = ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_uint8)
    D, I, M = int(n_groups), int(n_stages), int(n_micro)
    f = np.ascontiguousarray(f_cost, dtype=np.int32).reshape(-1)
    b = np.ascontiguousarray(b_cost, dtype=np.int32).reshape(-1)
    fs = np.ascontiguousarray(np.asarray(fail_stop, dtype=bool), dtype=np.uint8).reshape(-1)
    cap = np.ascontiguousarray(capacity, dtype=np.int32).reshape(-1)
    if not (f.size == b.size == fs.size == cap.size == D * I):
        raise ValueError("migration_plan_run: arrays must be [groups, stages]")
    asg = None
    if assignment is not None:
        asg = np.ascontiguousarray(assignment, dtype=np.int32).reshape(-1)
        if asg.size != D * M * I:
            raise ValueError("migration_plan_run: assignment must be [groups, micro, stages]")
    cap_moves = D * M * I if moves_capacity is None else int(moves_capacity)
    moves = (Move * max(cap_moves, 1))()
    makespan = np.zeros(D, dtype=np.int32)
    executed = np.full(D * M * I, -1, dtype=np.int32)
    n_moves, it_time = ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib().migration_plan_run(D, I, M, f.ctypes.data_as(i32p), b.ctypes.data_as(i32p),
                                  fs.ctypes.data_as(u8p), cap.ctypes.data_as(i32p), int(delta),
                                  int(p2p), 1 if migrate else 0,
                                  None if asg is None else asg.ctypes.data_as(i32p),
                                  makespan.ctypes.data_as(i32p), executed.ctypes.data_as(i32p),
                                  moves, cap_moves, ctypes.byref(n_moves), ctypes.byref(it_time))
    if rc == INVALID_ARG:
        raise ValueError("migration_plan_run: invalid argument")
    if rc != OK:
        raise RuntimeError(f"migration_plan_run: status {rc}")
    mv = [(m.slot, m.stage, m.source, m.destination, (m.group, m.micro_batch))
          for m in moves[:n_moves.value]]
    return {"iteration_time": int(it_time.value), "makespan": makespan.tolist(),
            "executed": executed.reshape(D, M, I), "migrations": mv}
