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


def test_reading_against_the_literal_listing():
    """The recorded reading (a fail-stop stage is never a destination, and is the source while it
    has pending work) against the listing taken literally (argmin / argmax over all groups):
    identical on every state without fail-stop stages, and on the fail-stop states the literal
    form either agrees or shows the two defects the reading avoids."""
    import itertools
    for n in (2, 3):
        for progress in itertools.product(range(3), repeat=n):
            for pend in itertools.product((None, 7), repeat=n):
                for mem in itertools.product((False, True), repeat=n):
                    for delta in (0, 1):
                        a = O.decide(list(progress), [False] * n, delta, list(pend), list(mem))
                        b = O.decide_literal(list(progress), [False] * n, delta, list(pend), list(mem))
                        assert a == b
    # the paper's own example is the same under both
    assert O.decide_literal([2, 1, 2], [False] * 3, 0, [None, 5, None], [True] * 3) == (1, 0, 5)
    # defect 1: a crashed stage that happens to be ahead is never d_min, its work stays put
    assert O.decide_literal([1, 5, 1], [False, True, False], 9, [None, 4, None], [True] * 3) is None
    assert O.decide([1, 5, 1], [False, True, False], 9, [None, 4, None], [True] * 3) == (1, 0, 4)
    # defect 2: a crashed stage with the largest count is taken as the destination
    assert O.decide_literal([0, 5, 1], [False, True, False], 0, [3, None, None], [True] * 3) == (0, 1, 3)
    assert O.decide([0, 5, 1], [False, True, False], 0, [3, None, None], [True] * 3) == (0, 2, 3)
