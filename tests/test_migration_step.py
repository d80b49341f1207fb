"""One migration decision of Algorithm 1 (host library) against the oracle on seeded states of
2 to 8 DP groups with fail-stop and lagging stages (Section 6.3), and its error paths."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import migration_step as O
from paper_2605_06374_amd import migration_step as M

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "migration_step.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(migration_step_[a-z_]+)\s*\(", text)))
    assert names == ["migration_step_decide"]
    assert hasattr(ctypes.CDLL(M.LIB_PATH), "migration_step_decide")


def test_worked_example_through_the_library():
    assert M.migration_step_decide([2, 1, 2], [False] * 3, 0, [None, 5, None], [True] * 3) == (1, 0, 5)


def test_matches_oracle_on_seeded_states():
    rng = np.random.default_rng(41)
    for trial in range(2000):
        n = int(rng.integers(1, 9))
        progress = rng.integers(0, 9, size=n).tolist()
        stop = (rng.random(n) < 0.15).tolist()
        pending = [None if rng.random() < 0.3 else int(rng.integers(0, 64)) for _ in range(n)]
        mem = (rng.random(n) < 0.8).tolist()
        delta = int(rng.integers(0, 3))
        assert M.migration_step_decide(progress, stop, delta, pending, mem) == \
            O.decide(progress, stop, delta, pending, mem)


def test_error_paths():
    with pytest.raises(ValueError):
        M.migration_step_decide([1, 2], [False, False], -1, [1, 2], [True, True])
    with pytest.raises(ValueError):
        M.migration_step_decide([1, 2], [False], 0, [1, 2], [True, True])
    assert M.lib().migration_step_decide(None, None, 2, 0, None, None, None, None, None) == M.INVALID_ARG
