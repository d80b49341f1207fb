"""Oracle (test infrastructure, CPU): the whole loop of Algorithm 1 (Section 6.3,
"Progress-Aware Workload Migration") around a slot-by-slot pipeline simulation.

What the section fixes: the loop ("while unfinished workloads exist: advance the pipeline
schedules; for every PP stage compute P_{d,i,t}, take d_min / d_max, and if (d_min, i) is
fail-stop or the gap exceeds delta move NextPending(d_min, i) to d_max when memory allows,
then update both P"), the meaning of P (forward workloads completed by stage i of group d,
local and migrated), the three constraints (every stage of every micro-batch runs exactly once;
dependencies are kept across the move; M <= C on the destination, activations live until their
backward completes) and the objective (the largest completion time over the DP groups).
What it leaves to a figure that the text does not hold, and is read here as follows:

  * time runs in unit slots; every (group, stage) is one executor that runs one chunk at a time;
  * chunks are F(d, j, i) and B(d, j, i) of micro-batch j of source group d at stage i (the W
    chunk of a stage follows its B on the same executor and has no successor: it is folded into
    B's cost); F(d, j, i) needs F(d, j, i - 1); B(d, j, i) needs B(d, j, i + 1) (the last stage:
    its own F) and runs where F(d, j, i) ran, because the activations live there; a chunk whose
    predecessor ran on another stage becomes ready `p2p` slots after it completed;
  * an idle executor runs a ready B if it has one (lowest (d, j) first), else the first ready F of
    its queue if an activation slot is free (one-forward-one-backward order), else nothing;
    its queue holds its own micro-batches in order, migrated ones behind them in arrival order;
  * memory: M_{e,i} = forwards started on executor (e, i) whose backward there has not completed;
    a forward only starts while M < C, so M <= C holds at every slot; MemoryFeasible(j, i, e) is
    M_{e,i} < C_{e,i} at the slot of the decision;
  * a fail-stop stage is known when the iteration starts and runs nothing in it;
  * NextPending(d, i): the first forward of stage i in d's queue that has not started;
  * "update P": the source is credited one forward (it has one fewer to do), the destination
    earns its credit when it completes the migrated forward;
  * T_makespan(d): the last slot in which an executor of group d completes a chunk.

The decision inside the loop is oracle/migration_step.decide.  Pins:
tests/test_oracle_pins_migration_plan.py.  Only tests, smoke() and bench.py's baseline leg may
import this."""
from __future__ import annotations

from . import migration_step


class Unschedulable(Exception):
    """Some workload can never run (e.g. a stage is fail-stop in every group)."""


def simulate(n_groups, n_stages, n_micro, f_cost, b_cost, fail_stop, capacity, delta, p2p=0,
             migrate=True, assignment=None, max_slots=None):
    """f_cost[e][i], b_cost[e][i]: slots per chunk on executor (e, i); fail_stop[e][i]: bool;
    capacity[e][i]: activation slots.  migrate=False: no decisions are taken (the plain schedule).
    assignment: optional {(d, j, i): e} fixed executor of every workload (used by the brute-force
    pins; implies migrate=False).  Returns a dict: iteration_time, makespan (per group),
    migrations [(slot, stage, source, destination, (d, j))], executed {(d, j, i): e},
    max_live (largest M seen per executor), done_f / done_b (completion slots)."""
    D, I, M = n_groups, n_stages, n_micro
    if assignment is not None:
        migrate = False
    if max_slots is None:
        worst = max(max(r) for r in f_cost) + max(max(r) for r in b_cost) + p2p
        max_slots = 4 * D * M * I * worst + 1000
    # queue[e][i]: forwards assigned to executor (e, i) that have not started, in order
    queue = [[[] for _ in range(I)] for _ in range(D)]
    for d in range(D):
        for j in range(M):
            for i in range(I):
                e = d if assignment is None else assignment[(d, j, i)]
                queue[e][i].append((d, j))
    owed_b = [[[] for _ in range(I)] for _ in range(D)]   # backwards an executor still has to run
    done_f, done_b, ran_on = {}, {}, {}
    busy_until = [[0] * I for _ in range(D)]
    running = [[None] * I for _ in range(D)]     # (kind, d, j) of the chunk in flight
    live = [[0] * I for _ in range(D)]
    max_live = [[0] * I for _ in range(D)]
    progress = [[0] * I for _ in range(D)]
    makespan = [0] * D
    migrations = []
    total = 2 * D * M * I
    t = 0
    while len(done_f) + len(done_b) < total:
        if t > max_slots:
            raise Unschedulable("slot limit reached: some workload can never run")
        # ---- advance the pipeline schedules: completions of this slot ...
        for e in range(D):
            for i in range(I):
                if running[e][i] is not None and busy_until[e][i] == t:
                    kind, d, j = running[e][i]
                    running[e][i] = None
                    makespan[e] = t
                    if kind == "F":
                        done_f[(d, j, i)] = t
                        progress[e][i] += 1
                        owed_b[e][i].append((d, j))
                    else:
                        done_b[(d, j, i)] = t
                        live[e][i] -= 1
        # ... then every idle executor starts what it can
        for e in range(D):
            for i in range(I):
                if running[e][i] is not None or fail_stop[e][i]:
                    continue
                pick = None
                for (d, j) in sorted(owed_b[e][i]):          # a ready backward first
                    if i == I - 1:
                        ready = done_f[(d, j, i)]
                    else:
                        ready = done_b[(d, j, i + 1)] + p2p if (d, j, i + 1) in done_b else None
                    if ready is not None and ready <= t:
                        pick = ("B", d, j)
                        break
                if pick is None and live[e][i] < capacity[e][i]:
                    for (d, j) in queue[e][i]:                # else the first ready forward
                        if i == 0:
                            ready = 0
                        else:
                            ready = done_f[(d, j, i - 1)] + p2p if (d, j, i - 1) in done_f else None
                        if ready is not None and ready <= t:
                            pick = ("F", d, j)
                            break
                if pick is None:
                    continue
                kind, d, j = pick
                running[e][i] = pick
                if kind == "F":
                    queue[e][i].remove((d, j))
                    ran_on[(d, j, i)] = e
                    live[e][i] += 1
                    max_live[e][i] = max(max_live[e][i], live[e][i])
                    busy_until[e][i] = t + f_cost[e][i]
                else:
                    owed_b[e][i].remove((d, j))
                    busy_until[e][i] = t + b_cost[e][i]
        # ---- one decision per stage
        if migrate:
            for i in range(I):
                pending = [queue[e][i][0] if queue[e][i] else None for e in range(D)]
                ids = [None if p is None else p[0] * M + p[1] for p in pending]
                feasible = [live[e][i] < capacity[e][i] for e in range(D)]
                got = migration_step.decide([progress[e][i] for e in range(D)],
                                            [fail_stop[e][i] for e in range(D)], delta, ids, feasible)
                if got is None:
                    continue
                src, dst, _ = got
                work = queue[src][i].pop(0)
                queue[dst][i].append(work)
                progress[src][i] += 1
                migrations.append((t, i, src, dst, work))
        t += 1
    return {"iteration_time": max(makespan), "makespan": makespan, "migrations": migrations,
            "executed": ran_on, "max_live": max_live, "done_f": done_f, "done_b": done_b}
