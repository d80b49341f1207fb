"""Oracle (test infrastructure, CPU): iteration-time prediction of Section 5.2, Eq. 2.

The pipeline schedule is a DAG: a vertex per computation chunk F(m,s), B(m,s), W(m,s) (forward,
backward-activation, backward-weight of micro-batch m at stage s) with its execution cost;
data edges F(m,s-1) -> F(m,s) and B(m,s+1) -> B(m,s) carry the point-to-point time, F(m,S-1) ->
B(m,S-1), F(m,s) -> B(m,s) and B(m,s) -> W(m,s) carry none; consecutive chunks of one stage, in
the order the schedule gives, are joined by zero-weight resource edges.  Eq. 2:
    t_start(v) = max over predecessors u of  t_start(u) + cost(u) + edge(u, v)
and the predicted healthy iteration time is the completion time of the last vertex.
Written as that definition: vertices are relaxed in a topological order found by repeated
scanning (no cleverness), in fp64.  Only tests, smoke() and bench.py's baseline leg may import
this module.

The two schedules named in Table 3 are built here as per-stage chunk orders:
* 1F1B: stage s runs min(S-1-s, M) warm-up forwards, then alternates one forward and one
  backward, then drains the backwards (the backward is one chunk: kinds F and B only);
* ZBH (reading: the handcrafted ZB-H1 schedule of the zero-bubble paper, memory of 1F1B): built
  by the rule "at every unit-cost time step a stage runs a ready B if there is one, else a ready
  F if fewer than S-s micro-batches are in flight on it, else a pending W".

Pins: tests/test_oracle_pins_pipeline_dag.py.
"""
from __future__ import annotations

F, B, W = 0, 1, 2


def schedule_1f1b(stages, microbatches):
    """Per-stage chunk order [(kind, m), ...] of the one-forward-one-backward schedule."""
    out = []
    for s in range(stages):
        warm = min(stages - 1 - s, microbatches)
        order = [(F, m) for m in range(warm)]
        for i in range(microbatches - warm):
            order += [(F, warm + i), (B, i)]
        order += [(B, i) for i in range(microbatches - warm, microbatches)]
        out.append(order)
    return out


def schedule_zbh1(stages, microbatches):
    """Per-stage chunk order with the backward split into B and W (see the module text)."""
    S, M = stages, microbatches
    done = {}                      # (kind, m, s) -> finish time (unit costs)
    order = [[] for _ in range(S)]
    nf = [0] * S; nb = [0] * S; nw = [0] * S
    t = 0
    while any(nw[s] < M for s in range(S)):
        started = []
        for s in range(S):
            pick = None
            if nb[s] < M:
                m = nb[s]
                dep = (B, m, s + 1) if s + 1 < S else (F, m, s)
                if done.get(dep, 1 << 60) <= t and done.get((F, m, s), 1 << 60) <= t:
                    pick = (B, m)
            if pick is None and nf[s] < M and nf[s] - nb[s] < S - s:
                m = nf[s]
                if s == 0 or done.get((F, m, s - 1), 1 << 60) <= t:
                    pick = (F, m)
            if pick is None and nw[s] < nb[s]:
                pick = (W, nw[s])
            if pick is not None:
                started.append((s, pick))
        for s, (kind, m) in started:
            order[s].append((kind, m))
            done[(kind, m, s)] = t + 1
            if kind == F: nf[s] += 1
            elif kind == B: nb[s] += 1
            else: nw[s] += 1
        t += 1
        if t > 16 * (M + S) + 16:
            raise RuntimeError("schedule construction does not terminate")
    return order


def simulate(stages, microbatches, schedule, cost, p2p):
    """Eq. 2.  cost[kind][m][s]; returns (iteration_time, {(kind, m, s): t_start})."""
    S, M = stages, microbatches
    preds = {}
    for s, order in enumerate(schedule):
        for pos, (kind, m) in enumerate(order):
            v = (kind, m, s)
            if v in preds:
                raise ValueError("chunk scheduled twice")
            p = []
            if pos > 0:
                pk, pm = order[pos - 1]
                p.append(((pk, pm, s), 0.0))
            if kind == F and s > 0:
                p.append(((F, m, s - 1), p2p))
            if kind == B:
                p.append(((F, m, s), 0.0))
                if s + 1 < S:
                    p.append(((B, m, s + 1), p2p))
            if kind == W:
                p.append(((B, m, s), 0.0))
            preds[v] = p
    for v, p in preds.items():
        for u, _ in p:
            if u not in preds:
                raise ValueError(f"chunk {v} depends on {u}, which the schedule does not hold")
    t_start = {}
    remaining = dict(preds)
    while remaining:
        progressed = False
        for v in list(remaining):
            p = remaining[v]
            if all(u in t_start for u, _ in p):
                t_start[v] = max([t_start[u] + cost[u[0]][u[1]][u[2]] + e for u, e in p], default=0.0)
                del remaining[v]
                progressed = True
        if not progressed:
            raise ValueError("the schedule order contradicts the data dependencies (cycle)")
    total = max(t_start[v] + cost[v[0]][v[1]][v[2]] for v in t_start)
    return total, t_start
