"""TP subgroup selection (host library) against the oracle on seeded TP groups of 1 to 16
devices with fail-stop and fail-slow members (Section 6.1), and its error paths."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import tp_select as O
from paper_2605_06374_amd import tp_select as T

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    text = open(os.path.join(ROOT, "include", "tp_select.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(tp_select_[a-z_]+)\s*\(", text)))
    assert names == ["tp_select_subgroup"]
    assert hasattr(ctypes.CDLL(T.LIB_PATH), "tp_select_subgroup")


def test_matches_oracle_on_seeded_groups():
    rng = np.random.default_rng(23)
    for trial in range(500):
        n = int(rng.choice([1, 2, 4, 8, 8, 8, 16, 5, 7]))
        # mostly healthy devices, some fail-slow at 20-90 %, ties on purpose (two decimals)
        p = np.where(rng.random(n) < 0.7, 1.0, np.round(rng.uniform(0.2, 0.9, size=n), 2))
        stop = [i for i in range(n) if rng.random() < 0.15]
        k_min = int(rng.choice([1, 2, 4]))
        want = O.select(p.tolist(), stop, k_min)
        got = T.tp_select_subgroup(p, stop, k_min)
        assert got[0] == want[0] and got[1] == want[1] and got[2] == want[2]
        assert abs(got[3] - want[3]) <= 1e-12


def test_paper_scale_example_group_of_eight():
    p = [1.0, 1.0, 0.4, 1.0, 1.0, 1.0, 1.0, 1.0]
    assert T.tp_select_subgroup(p, [], 1) == (4, [0, 1, 3, 4], [2, 5, 6, 7], 4.0)
    assert T.tp_select_subgroup(p, [], 8)[0] == 8
    assert T.tp_select_subgroup([1.0, 1.0], [0], 2) == (0, [], [1], 0.0)


def test_error_paths():
    with pytest.raises(ValueError):
        T.tp_select_subgroup([1.0, float("nan")], [], 1)
    with pytest.raises(ValueError):
        T.tp_select_subgroup([1.0, -0.1], [], 1)
    with pytest.raises(ValueError):
        T.tp_select_subgroup([1.0] * 65, [], 1)
    with pytest.raises(ValueError):
        T.tp_select_subgroup([1.0] * 4, [], 0)
    assert T.lib().tp_select_subgroup(None, None, 4, 1, None, None, None) == T.INVALID_ARG
    # a non-finite throughput on a fail-stop device is ignored
    assert T.tp_select_subgroup([float("nan"), 1.0], [0], 1) == (1, [1], [], 1.0)
