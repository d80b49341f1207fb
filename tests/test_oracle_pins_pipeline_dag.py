"""Pins of the iteration-time oracle (Section 5.2, Eq. 2): closed forms, an independent
event-driven simulation, and invariants of the start times."""
import itertools

import numpy as np
import pytest

from oracle import pipeline_dag as O

F, B, W = O.F, O.B, O.W


def uniform(kinds, M, S, values):
    return [[[values[k]] * S for _ in range(M)] for k in range(kinds)]


@pytest.mark.parametrize("S,M", [(1, 1), (2, 2), (4, 4), (4, 8), (8, 8), (3, 7), (8, 4)])
def test_1f1b_uniform_costs_closed_form(S, M):
    """Uniform costs and free communication: (M + S - 1) (F + B)."""
    f, b = 1.25, 2.5
    total, _ = O.simulate(S, M, O.schedule_1f1b(S, M), uniform(2, M, S, [f, b]), 0.0)
    assert abs(total - (M + S - 1) * (f + b)) < 1e-12


def test_single_stage_is_the_sum_and_single_microbatch_is_the_chain():
    rng = np.random.default_rng(3)
    M = 5
    cost = [[[float(rng.integers(1, 9))] for _ in range(M)] for _ in range(2)]
    total, _ = O.simulate(1, M, O.schedule_1f1b(1, M), cost, 0.7)
    assert total == sum(c[0] for k in cost for c in k)
    S = 6
    cost = [[[float(rng.integers(1, 9)) for _ in range(S)]] for _ in range(2)]
    total, _ = O.simulate(S, 1, O.schedule_1f1b(S, 1), cost, 0.5)
    assert total == sum(cost[0][0]) + sum(cost[1][0]) + 2 * (S - 1) * 0.5


@pytest.mark.parametrize("S,M", [(2, 2), (2, 5), (4, 4), (4, 8), (8, 8), (8, 16), (3, 9)])
def test_zbh1_uniform_costs_reach_the_published_bubble(S, M):
    """Zero-bubble paper, ZB-H1: bubble (S - 1)(T_F + T_B - T_W); with equal chunk times the
    iteration takes 3 M + S - 1 units."""
    sched = O.schedule_zbh1(S, M)
    for s, order in enumerate(sched):
        assert sorted(order) == sorted((k, m) for k in (F, B, W) for m in range(M))
        inflight, peak = 0, 0
        for k, m in order:
            inflight += (k == F) - (k == B)
            peak = max(peak, inflight)
        assert peak <= S - s          # activation memory of 1F1B
    total, _ = O.simulate(S, M, sched, uniform(3, M, S, [1.0, 1.0, 1.0]), 0.0)
    assert total == 3 * M + S - 1


def event_driven(S, M, schedule, cost, p2p):
    """Independent check: advance a clock; every stage runs its list in order and starts the
    next chunk as soon as the chunk's inputs have arrived."""
    finish, pos, free_at = {}, [0] * S, [0.0] * S

    def ready_time(kind, m, s):
        deps = []
        if kind == F and s > 0: deps.append(((F, m, s - 1), p2p))
        if kind == B:
            deps.append(((F, m, s), 0.0))
            if s + 1 < S: deps.append(((B, m, s + 1), p2p))
        if kind == W: deps.append(((B, m, s), 0.0))
        if any(d not in finish for d, _ in deps): return None
        return max([finish[d] + e for d, e in deps], default=0.0)

    while any(pos[s] < len(schedule[s]) for s in range(S)):
        moved = False
        for s in range(S):
            if pos[s] == len(schedule[s]): continue
            kind, m = schedule[s][pos[s]]
            r = ready_time(kind, m, s)
            if r is None: continue
            start = max(r, free_at[s])
            finish[(kind, m, s)] = free_at[s] = start + cost[kind][m][s]
            pos[s] += 1
            moved = True
        assert moved, "deadlock"
    return max(finish.values())


@pytest.mark.parametrize("builder,kinds", [(O.schedule_1f1b, 2), (O.schedule_zbh1, 3)])
def test_random_costs_match_event_driven_simulation(builder, kinds):
    rng = np.random.default_rng(17)
    for S, M in itertools.product((1, 2, 3, 5), (1, 2, 4, 7)):
        cost = [[[float(rng.integers(1, 20)) for _ in range(S)] for _ in range(M)] for _ in range(kinds)]
        p2p = float(rng.integers(0, 4))
        sched = builder(S, M)
        total, t_start = O.simulate(S, M, sched, cost, p2p)
        assert total == event_driven(S, M, sched, cost, p2p)
        # no stage runs two chunks at once, and the order of the schedule is kept
        for s, order in enumerate(sched):
            for (k0, m0), (k1, m1) in zip(order, order[1:]):
                assert t_start[(k1, m1, s)] >= t_start[(k0, m0, s)] + cost[k0][m0][s]


def test_slow_microbatch_moves_the_prediction_by_its_critical_share():
    """One longer micro-batch on every stage (a long document): with 1F1B, S = 2, M = 2 the
    critical path is F(0,0) F(0,1) B(0,1) F(1,1) B(1,1) B(1,0) by hand."""
    cost = [[[1.0, 1.0], [3.0, 3.0]], [[2.0, 2.0], [6.0, 6.0]]]
    total, _ = O.simulate(2, 2, O.schedule_1f1b(2, 2), cost, 0.0)
    # stage 1: F0 at 1..2, B0 2..4; F1 arrives at 1+3=4: 4..7, B1 7..13; stage 0: B1 13..19
    assert total == 19.0


def test_contradictory_schedule_is_refused():
    with pytest.raises(ValueError):
        O.simulate(2, 1, [[(B, 0), (F, 0)], [(F, 0), (B, 0)]], uniform(2, 1, 2, [1.0, 1.0]), 0.0)
    with pytest.raises(ValueError):
        O.simulate(2, 1, [[(F, 0), (B, 0)], [(F, 0)]], uniform(2, 1, 2, [1.0, 1.0]), 0.0)
