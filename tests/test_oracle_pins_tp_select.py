"""Pins of the TP subgroup selection oracle (Section 6.1, Eq. 3 and Eq. 4)."""
import itertools

import numpy as np

from oracle import tp_select as O


def test_feasible_degrees_by_hand():
    assert O.feasible_degrees(8, 1) == [1, 2, 4, 8]
    assert O.feasible_degrees(7, 2) == [2, 4]
    assert O.feasible_degrees(3, 4) == []
    assert O.feasible_degrees(1, 1) == [1]


def test_hand_cases():
    # all healthy, one fail-stop of eight: the largest power of two that fits is 4
    k, members, standby, value = O.select([1.0] * 8, [3], 1)
    assert k == 4 and value == 4.0 and 3 not in members + standby and len(standby) == 3
    # one device at 40 %: 8 * 0.4 = 3.2 < 4 * 1.0 -> the slow device is left out
    p = [1.0, 1.0, 0.4, 1.0, 1.0, 1.0, 1.0, 1.0]
    k, members, standby, value = O.select(p, [], 1)
    assert (k, value) == (4, 4.0) and 2 in standby and members == [0, 1, 3, 4]
    # at 60 % it is kept: 8 * 0.6 = 4.8 > 4
    p[2] = 0.6
    k, members, standby, value = O.select(p, [], 1)
    assert k == 8 and abs(value - 4.8) < 1e-12 and standby == []
    # memory bound forces degree 8 although 4 would be faster
    p[2] = 0.4
    assert O.select(p, [], 8)[0] == 8
    # nothing feasible
    assert O.select([1.0, 1.0], [0], 2) == (0, [], [1], 0.0)


def test_exhaustive_search_over_all_subsets_agrees():
    """Eq. 4 restricted to top-k candidates loses nothing: no subset of a feasible size has a
    larger k * min p."""
    rng = np.random.default_rng(5)
    for trial in range(300):
        n = int(rng.integers(1, 9))
        p = [float(x) for x in np.round(rng.uniform(0.05, 1.0, size=n), 2)]
        stop = [i for i in range(n) if rng.random() < 0.2]
        k_min = int(rng.choice([1, 1, 2, 4]))
        alive = [i for i in range(n) if i not in stop]
        best = 0.0
        for k in O.feasible_degrees(len(alive), k_min):
            for sub in itertools.combinations(alive, k):
                best = max(best, k * min(p[i] for i in sub))
        k, members, standby, value = O.select(p, stop, k_min)
        assert abs(value - best) < 1e-12
        if k:
            assert len(members) == k and abs(k * min(p[i] for i in members) - value) < 1e-12
            assert sorted(members + standby) == alive
            assert min(p[i] for i in members) >= max([p[i] for i in standby], default=0.0)
