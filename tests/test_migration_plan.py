"""The migration loop of Algorithm 1 (host library) against the oracle on seeded instances with
fail-slow and fail-stop stages (Section 6.3): identical moves, completion times and executors;
static plans; error paths."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import migration_plan as O
from paper_2605_06374_amd import migration_plan as M

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "migration_plan.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(migration_plan_[a-z_]+)\s*\(", text)))
    assert names == ["migration_plan_run"]
    assert hasattr(ctypes.CDLL(M.LIB_PATH), "migration_plan_run")
    assert ctypes.sizeof(M.Move) == 24


def instance(rng):
    D, I, Mb = int(rng.integers(1, 6)), int(rng.integers(1, 5)), int(rng.integers(1, 9))
    f = rng.integers(1, 4, size=(D, I))
    b = rng.integers(1, 6, size=(D, I))
    if rng.random() < 0.5:      # one slow stage
        f[rng.integers(0, D), rng.integers(0, I)] *= 3
    fs = np.zeros((D, I), dtype=bool)
    if D > 1 and rng.random() < 0.4:   # one crashed stage (never the same stage in all groups)
        fs[rng.integers(0, D), rng.integers(0, I)] = True
    cap = rng.integers(1, I + 4, size=(D, I))
    return D, I, Mb, f.tolist(), b.tolist(), fs.tolist(), cap.tolist(), int(rng.integers(0, 3)), int(rng.integers(0, 3))


def same(got, want, D, I, Mb):
    assert got["iteration_time"] == want["iteration_time"]
    assert got["makespan"] == want["makespan"]
    assert got["migrations"] == want["migrations"]
    for (d, j, i), e in want["executed"].items():
        assert int(got["executed"][d, j, i]) == e
    assert (got["executed"] >= 0).all()


def test_matches_oracle_on_seeded_instances():
    rng = np.random.default_rng(63)
    moved = 0
    for trial in range(300):
        D, I, Mb, f, b, fs, cap, delta, p2p = instance(rng)
        want = O.simulate(D, I, Mb, f, b, fs, cap, delta, p2p=p2p)
        got = M.migration_plan_run(D, I, Mb, f, b, fs, cap, delta, p2p=p2p)
        same(got, want, D, I, Mb)
        moved += len(want["migrations"])
        # the untouched schedule (only where no stage has crashed: its work could not run)
        if not np.any(fs):
            same(M.migration_plan_run(D, I, Mb, f, b, fs, cap, delta, p2p=p2p, migrate=False),
                 O.simulate(D, I, Mb, f, b, fs, cap, delta, p2p=p2p, migrate=False), D, I, Mb)
    assert moved > 200


def test_static_plans_match_oracle():
    rng = np.random.default_rng(64)
    for trial in range(100):
        D, I, Mb, f, b, fs, cap, delta, p2p = instance(rng)
        fs = [[False] * I for _ in range(D)]
        asg = rng.integers(0, D, size=(D, Mb, I))
        want = O.simulate(D, I, Mb, f, b, fs, cap, delta, p2p=p2p,
                          assignment={(d, j, i): int(asg[d, j, i]) for d in range(D) for j in range(Mb)
                                      for i in range(I)})
        got = M.migration_plan_run(D, I, Mb, f, b, fs, cap, delta, p2p=p2p, assignment=asg)
        same(got, want, D, I, Mb)


def test_worked_state_of_section_6_3_inside_the_loop():
    """Three groups, one stage, the middle group twice as slow: at the slot where the others have
    completed one forward more than it, its next pending micro-batch leaves for a fastest group
    (the lowest index of the tie), as in the section's example."""
    got = M.migration_plan_run(3, 1, 3, [[1], [2], [1]], [[1], [2], [1]], [[False]] * 3, [[9]] * 3, 0)
    first = got["migrations"][0]
    assert first[1:4] == (0, 1, 0) and first[4][0] == 1


def test_error_paths():
    ok = dict(n_groups=2, n_stages=2, n_micro=2, f_cost=[[1, 1], [1, 1]], b_cost=[[1, 1], [1, 1]],
              fail_stop=[[False, False]] * 2, capacity=[[2, 2]] * 2, delta=0)
    M.migration_plan_run(**ok)
    for key, bad in (("delta", -1), ("f_cost", [[0, 1], [1, 1]]), ("capacity", [[0, 2], [2, 2]]),
                     ("b_cost", [[1, 1]])):
        with pytest.raises(ValueError):
            M.migration_plan_run(**{**ok, key: bad})
    with pytest.raises(ValueError):
        M.migration_plan_run(**ok, assignment=[[[0, 2], [0, 0]], [[1, 1], [1, 1]]])
    # a stage that has crashed in every group: the work can never run
    with pytest.raises(RuntimeError):
        M.migration_plan_run(**{**ok, "fail_stop": [[True, False], [True, False]]})
    # more moves than the caller's array holds
    with pytest.raises(RuntimeError):
        M.migration_plan_run(**{**ok, "f_cost": [[5, 5], [1, 1]], "n_micro": 6}, moves_capacity=1)
    assert M.lib().migration_plan_run(0, 1, 1, None, None, None, None, 0, 0, 1, None, None, None, None,
                                      0, None, None) == M.INVALID_ARG
