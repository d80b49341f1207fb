"""Pins of the migration decision oracle (Section 6.3, Algorithm 1)."""
from oracle import migration_step as O


def test_worked_example_of_section_6_3():
    """Stage 0 at time slot T2: P_0 = P_2 = 2, P_1 = 1, delta = 0: the gap 2 - 1 = 1 > 0 makes
    DP1 the straggler and its pending forward of micro-batch 5 moves to a fastest group (DP0
    and DP2 tie; the lowest index is taken)."""
    assert O.decide([2, 1, 2], [False] * 3, 0, [None, 5, None], [True] * 3) == (1, 0, 5)
    # if DP0 cannot hold it, nothing moves in this slot (the algorithm looks at d_max only)
    assert O.decide([2, 1, 2], [False] * 3, 0, [None, 5, None], [False, True, True]) is None
    # with delta = 1 the same gap is tolerated
    assert O.decide([2, 1, 2], [False] * 3, 1, [None, 5, None], [True] * 3) is None


def test_fail_stop_eviction():
    """A crashed stage hands its pending micro-batches to a healthy peer whatever the gap."""
    assert O.decide([3, 3, 3], [False, True, False], 5, [7, 4, 8], [True] * 3) == (1, 0, 4)
    assert O.decide([3, 9, 4], [False, True, False], 5, [7, 4, 8], [True] * 3) == (1, 2, 4)
    # nothing pending on the crashed stage: ordinary balancing among the healthy groups
    assert O.decide([1, 0, 4], [False, True, False], 2, [7, None, 8], [True] * 3) == (0, 2, 7)
    assert O.decide([0, 0], [True, True], 0, [1, 2], [True, True]) is None


def test_no_self_migration_and_no_pending():
    assert O.decide([2, 2, 2], [False] * 3, 0, [1, 2, 3], [True] * 3) is None
    assert O.decide([5, 1], [False, False], 0, [None, None], [True, True]) is None
    assert O.decide([4], [False], 0, [9], [True]) is None
