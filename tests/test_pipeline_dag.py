"""Iteration-time predictor (host library) against the oracle: schedules identical chunk by
chunk, start times and iteration time equal on seeded costs shaped like Table 3's settings
(4-8 micro-batches, 2-16 stages, per-micro-batch costs from Eq. 1 on packed lengths)."""
import ctypes
import itertools
import os
import re

import numpy as np
import pytest

from oracle import mb_time as OT
from oracle import pipeline_dag as O
from paper_2605_06374_amd import pipeline_dag as P
from paper_2605_06374_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "pipeline_dag.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(pipeline_dag_[a-z0-9_]+)\s*\(", text)))
    assert {"pipeline_dag_schedule_1f1b", "pipeline_dag_schedule_zbh1",
            "pipeline_dag_simulate"} <= set(names)
    lib = ctypes.CDLL(P.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert ctypes.sizeof(P.Chunk) == 8


@pytest.mark.parametrize("S,M", list(itertools.product((1, 2, 3, 4, 8, 16), (1, 2, 4, 8, 13))))
def test_schedules_equal_the_oracles(S, M):
    assert P.pipeline_dag_schedule_1f1b(S, M) == O.schedule_1f1b(S, M)
    assert P.pipeline_dag_schedule_zbh1(S, M) == O.schedule_zbh1(S, M)


def eq1_costs(kinds, S, M, seed):
    """Chunk costs from Eq. 1 on packed micro-batches of the length-skew sweep: F = alpha N +
    beta sum l^2 per stage, B = 2 F (or B = W = F when split), stages a few percent apart."""
    rng = np.random.default_rng(seed)
    feats = [OT.tokens_and_sum_sq(W.config(5, microbatch=int(i)).cu_seqlens)
             for i in rng.integers(0, 64, size=M)]
    stage_scale = 1.0 + 0.05 * rng.standard_normal(S)
    f = np.array([[(0.4 * n + 3e-5 * q) * stage_scale[s] for s in range(S)] for n, q in feats])
    return np.stack([f, 2.0 * f] if kinds == 2 else [f, f, f])


@pytest.mark.parametrize("builder,kinds", [("1f1b", 2), ("zbh1", 3)])
def test_simulation_matches_oracle(builder, kinds):
    for idx, (S, M) in enumerate(itertools.product((1, 2, 4, 8, 16), (1, 4, 8))):
        cost = eq1_costs(kinds, S, M, 100 + idx)
        p2p = 35.0
        sched = getattr(O, "schedule_" + builder)(S, M)
        want_total, want_start = O.simulate(S, M, sched, cost.tolist(), p2p)
        total, starts = P.pipeline_dag_simulate(S, M, sched, cost, p2p, want_starts=True)
        assert abs(total - want_total) <= 1e-9 * want_total
        for (k, m, s), t in want_start.items():
            assert abs(starts[k, m, s] - t) <= 1e-9 * max(1.0, t)


def test_closed_forms_through_the_library():
    S, M = 8, 8
    c = np.stack([np.full((M, S), 1.5), np.full((M, S), 3.0)])
    assert P.pipeline_dag_simulate(S, M, P.pipeline_dag_schedule_1f1b(S, M), c, 0.0) == (M + S - 1) * 4.5
    c = np.ones((3, M, S))
    assert P.pipeline_dag_simulate(S, M, P.pipeline_dag_schedule_zbh1(S, M), c, 0.0) == 3 * M + S - 1


def test_error_paths():
    ones = np.ones((2, 1, 2))
    with pytest.raises(ValueError):   # order contradicts the dependencies
        P.pipeline_dag_simulate(2, 1, [[(P.B, 0), (P.F, 0)], [(P.F, 0), (P.B, 0)]], ones, 0.0)
    with pytest.raises(ValueError):   # a chunk twice
        P.pipeline_dag_simulate(2, 1, [[(P.F, 0), (P.F, 0)], [(P.F, 0), (P.B, 0)]], ones, 0.0)
    with pytest.raises(ValueError):   # bad kind
        P.pipeline_dag_simulate(2, 1, [[(P.F, 0), (P.W, 0)], [(P.F, 0), (P.B, 0)]], ones, 0.0)
    with pytest.raises(ValueError):   # negative cost
        P.pipeline_dag_simulate(2, 1, O.schedule_1f1b(2, 1), -ones, 0.0)
    with pytest.raises(ValueError):
        P.pipeline_dag_schedule_1f1b(0, 4)
    lib = P.lib()
    assert lib.pipeline_dag_simulate(2, 1, 2, None, None, 0.0, None, None) == P.INVALID_ARG
