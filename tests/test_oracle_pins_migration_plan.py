"""Pins of the migration-loop oracle (Section 6.3, Algorithm 1 with the slot simulation around
it).  The paper prints no schedule for it (its figure is not in the text), so the pins are what
the section's problem statement and the mathematics fix: the untouched schedule equals the
one-forward-one-backward closed form and the DAG predictor of Section 5.2 (Eq. 2); completeness,
dependencies and the memory bound hold on every run; a fail-stop stage runs nothing; and on tiny
instances the heuristic lies between the best static plan (brute force over all of them) and the
untouched schedule."""
import itertools

import numpy as np
import pytest

from oracle import migration_plan as P
from oracle import pipeline_dag as DAG


def uniform(D, I, f=1, b=2):
    return [[f] * I for _ in range(D)], [[b] * I for _ in range(D)]


def check_run(r, D, I, M, f_cost, b_cost, fail_stop, capacity, p2p):
    """Constraints (1)-(3) of the section on a finished run."""
    # (1) every stage of every micro-batch ran exactly once, on a healthy executor
    assert sorted(r["executed"]) == [(d, j, i) for d in range(D) for j in range(M) for i in range(I)]
    assert len(r["done_f"]) == len(r["done_b"]) == D * M * I
    for (d, j, i), e in r["executed"].items():
        assert not fail_stop[e][i]
    # (2) dependencies, with the exchange time between stages
    for (d, j, i), e in r["executed"].items():
        start_f = r["done_f"][(d, j, i)] - f_cost[e][i]
        start_b = r["done_b"][(d, j, i)] - b_cost[e][i]
        if i > 0:
            assert start_f >= r["done_f"][(d, j, i - 1)] + p2p
        if i < I - 1:
            assert start_b >= r["done_b"][(d, j, i + 1)] + p2p
        assert start_b >= r["done_f"][(d, j, i)]
    # one chunk at a time per executor
    for e in range(D):
        for i in range(I):
            spans = []
            for (d, j, s), ex in r["executed"].items():
                if s == i and ex == e:
                    spans.append((r["done_f"][(d, j, i)] - f_cost[e][i], r["done_f"][(d, j, i)]))
                    spans.append((r["done_b"][(d, j, i)] - b_cost[e][i], r["done_b"][(d, j, i)]))
            spans.sort()
            for (a0, a1), (b0, b1) in zip(spans, spans[1:]):
                assert a1 <= b0
    # (3) activations never exceed the capacity: recount from the spans
    for e in range(D):
        for i in range(I):
            events = []
            for (d, j, s), ex in r["executed"].items():
                if s == i and ex == e:
                    events.append((r["done_f"][(d, j, i)] - f_cost[e][i], 1))
                    events.append((r["done_b"][(d, j, i)], -1))
            live = worst = 0
            for _, delta in sorted(events, key=lambda x: (x[0], x[1])):
                live += delta
                worst = max(worst, live)
            assert worst <= capacity[e][i] and worst == r["max_live"][e][i]
    # completion times
    for e in range(D):
        mine = [r["done_b"][k] for k, ex in r["executed"].items() if ex == e] + \
               [r["done_f"][k] for k, ex in r["executed"].items() if ex == e]
        assert r["makespan"][e] == (max(mine) if mine else 0)
    assert r["iteration_time"] == max(r["makespan"])


@pytest.mark.parametrize("D,I,M,f,b", [(1, 1, 1, 1, 1), (2, 3, 4, 1, 2), (3, 4, 8, 2, 3), (2, 5, 5, 1, 1)])
def test_untouched_schedule_is_one_forward_one_backward(D, I, M, f, b):
    """Healthy, equal groups whose stages hold the activations 1F1B keeps in flight (I - i at
    stage i): no gap ever opens, nothing moves, and the iteration takes (M + I - 1) (F + B) slots,
    the closed form of 1F1B; the DAG predictor of Section 5.2 gives the same number for the same
    chunk times (W folded into B)."""
    fc, bc = uniform(D, I, f, b)
    cap = [[I - i for i in range(I)] for _ in range(D)]
    r = P.simulate(D, I, M, fc, bc, [[False] * I] * D, cap, 0)
    assert r["migrations"] == []
    assert r["iteration_time"] == (M + I - 1) * (f + b)
    assert r["makespan"] == [(M + I - 1) * (f + b)] * D
    cost = {DAG.F: [[float(f)] * I for _ in range(M)], DAG.B: [[float(b)] * I for _ in range(M)]}
    t, _ = DAG.simulate(I, M, DAG.schedule_1f1b(I, M), cost, 0.0)
    assert t == r["iteration_time"]
    check_run(r, D, I, M, fc, bc, [[False] * I] * D, cap, 0)


def test_exchange_time_between_stages():
    fc, bc = uniform(1, 3, 1, 1)
    r = P.simulate(1, 3, 1, fc, bc, [[False] * 3], [[3] * 3], 0, p2p=2)
    assert r["iteration_time"] == 6 + 4 * 2     # six chunks and four hops
    check_run(r, 1, 3, 1, fc, bc, [[False] * 3], [[3] * 3], 2)


def test_fail_stop_stage_is_emptied():
    D, I, M = 3, 3, 4
    fc, bc = uniform(D, I)
    fs = [[False] * I for _ in range(D)]
    fs[1][2] = True
    cap = [[I + 2] * I for _ in range(D)]
    r = P.simulate(D, I, M, fc, bc, fs, cap, delta=1)
    moved = [m for m in r["migrations"] if m[1] == 2 and m[2] == 1]
    assert sorted(m[4] for m in moved) == [(1, j) for j in range(M)]      # every workload of the stage
    assert all(m[3] in (0, 2) for m in moved)
    check_run(r, D, I, M, fc, bc, fs, cap, 0)
    # the same stage down in every group: nothing can run it
    fs_all = [[False, False, True] for _ in range(D)]
    with pytest.raises(P.Unschedulable):
        P.simulate(D, I, M, fc, bc, fs_all, cap, delta=1)


def test_straggler_is_relieved_and_constraints_hold():
    rng = np.random.default_rng(3)
    for trial in range(40):
        D, I, M = int(rng.integers(2, 5)), int(rng.integers(1, 4)), int(rng.integers(2, 7))
        fc = [[1] * I for _ in range(D)]
        bc = [[2] * I for _ in range(D)]
        slow = int(rng.integers(0, D))
        k = int(rng.integers(2, 5))
        st = int(rng.integers(0, I))
        fc[slow][st], bc[slow][st] = k, 2 * k
        cap = [[int(rng.integers(1, I + 3)) for _ in range(I)] for _ in range(D)]
        fs = [[False] * I for _ in range(D)]
        delta = int(rng.integers(0, 3))
        p2p = int(rng.integers(0, 2))
        r = P.simulate(D, I, M, fc, bc, fs, cap, delta, p2p=p2p)
        check_run(r, D, I, M, fc, bc, fs, cap, p2p)
        base = P.simulate(D, I, M, fc, bc, fs, cap, delta, p2p=p2p, migrate=False)
        check_run(base, D, I, M, fc, bc, fs, cap, p2p)
        assert base["migrations"] == []
        # moves only ever leave the group that is behind at that stage
        assert all(m[2] != m[3] for m in r["migrations"])


@pytest.mark.parametrize("D,I,M", [(2, 1, 3), (2, 2, 2), (3, 1, 2)])
def test_between_the_best_static_plan_and_the_untouched_schedule(D, I, M):
    """Brute force over every static plan x (the executor of every (micro-batch, stage)), run by
    the same executors: the heuristic can be no better than the best of them and, with one slow
    group and ample memory, is no worse than leaving everything in place."""
    fc = [[1] * I for _ in range(D)]
    bc = [[1] * I for _ in range(D)]
    fc[0] = [3] * I
    bc[0] = [3] * I
    fs = [[False] * I for _ in range(D)]
    cap = [[D * M] * I for _ in range(D)]
    keys = [(d, j, i) for d in range(D) for j in range(M) for i in range(I)]
    best = None
    for choice in itertools.product(range(D), repeat=len(keys)):
        t = P.simulate(D, I, M, fc, bc, fs, cap, 0, assignment=dict(zip(keys, choice)))["iteration_time"]
        best = t if best is None else min(best, t)
    heuristic = P.simulate(D, I, M, fc, bc, fs, cap, 0)["iteration_time"]
    untouched = P.simulate(D, I, M, fc, bc, fs, cap, 0, migrate=False)["iteration_time"]
    assert best <= heuristic <= untouched
    assert heuristic < untouched           # the slow group is relieved
    print(f"D={D} I={I} M={M}: best static {best}, heuristic {heuristic}, untouched {untouched}")
