"""Oracle (test infrastructure, CPU): one scheduling decision of Algorithm 1 (Section 6.3).

For one PP stage i at one time slot, given the progress P_d (forward workloads completed by
stage i in DP group d, local and migrated), which groups are fail-stop at this stage, the
threshold delta, the next pending micro-batch of every group at this stage (None if none) and
whether the destination could hold it (memory):
  1. d_min = argmin_d P_d, d_max = argmax_d P_d;
  2. a migration is wanted if (d_min, i) is fail-stop or P_dmax - P_dmin > delta;
  3. the next pending micro-batch j of d_min moves to d_max if j exists and is memory-feasible
     there.
Readings: a fail-stop group is never a destination and is always the source while it has
pending work (lowest index first); ties of argmin / argmax go to the lowest index; a group is
not its own destination.  Only tests, smoke() and bench.py's baseline leg may import this.

Pins: tests/test_oracle_pins_migration_step.py (the worked example of Section 6.3).
"""
from __future__ import annotations


def decide(progress, fail_stop, delta, next_pending, memory_feasible):
    """Returns (source, destination, micro_batch) or None."""
    groups = range(len(progress))
    stopped = [d for d in groups if fail_stop[d]]
    healthy = [d for d in groups if not fail_stop[d]]
    if not healthy:
        return None
    d_max = max(healthy, key=lambda d: (progress[d], -d))
    sources = [d for d in stopped if next_pending[d] is not None]
    if sources:
        d_min, wanted = sources[0], True
    else:
        d_min = min(healthy, key=lambda d: (progress[d], d))
        wanted = progress[d_max] - progress[d_min] > delta
    if not wanted or d_min == d_max:
        return None
    j = next_pending[d_min]
    if j is None or not memory_feasible[d_max]:
        return None
    return d_min, d_max, j


def decide_literal(progress, fail_stop, delta, next_pending, memory_feasible):
    """The listing of Algorithm 1 taken literally: argmin and argmax over ALL groups (ties to the
    lowest index), the test "(d_min, i) is fail-stop or the gap exceeds delta", NextPending of
    d_min, MemoryFeasible of d_max.  Kept beside `decide` so that the tests can show where the
    recorded reading departs from the listing: a fail-stop group that is ahead of the others is
    never d_min here, so its pending work would stay where it cannot run, and a fail-stop group
    can be d_max, i.e. a destination."""
    groups = range(len(progress))
    d_min = min(groups, key=lambda d: (progress[d], d))
    d_max = max(groups, key=lambda d: (progress[d], -d))
    if not (fail_stop[d_min] or progress[d_max] - progress[d_min] > delta):
        return None
    j = next_pending[d_min]
    if j is None or not memory_feasible[d_max] or d_min == d_max:
        return None
    return d_min, d_max, j
