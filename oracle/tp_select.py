"""Oracle (test infrastructure, CPU): selective device exclusion inside a TP group, Section 6.1.

G is the original TP group, F_stop its fail-stop devices, G' = G \\ F_stop.  Feasible degrees
(Eq. 3): K = {k : k_min <= k <= |G'|, k a power of two}.  For each k the candidate S_k is the
top-k devices of G' by normalised throughput p_i, and the choice (Eq. 4) is
    S* = argmax over k in K of  k * min_{i in S_k} p_i .
Devices of G' outside S* stay online as standby.  Written as those definitions.  Readings: ties
between degrees go to the larger degree; ties between devices go to the lower index.  Only
tests, smoke() and bench.py's baseline leg may import this module.

Pins: tests/test_oracle_pins_tp_select.py (exhaustive search over every subset of G' of a
feasible size, hand cases).
"""
from __future__ import annotations


def feasible_degrees(n_alive, k_min):
    """Eq. 3."""
    out, k = [], 1
    while k <= n_alive:
        if k >= k_min:
            out.append(k)
        k *= 2
    return out


def select(p, fail_stop, k_min):
    """p: normalised throughput per device of G (index = position in G); fail_stop: indices.
    Returns (degree, members sorted by index, standby sorted by index, k * min p), or
    (0, [], alive, 0.0) when no feasible degree exists."""
    stop = set(int(i) for i in fail_stop)
    alive = [i for i in range(len(p)) if i not in stop]
    ranked = sorted(alive, key=lambda i: (-float(p[i]), i))
    best = None
    for k in feasible_degrees(len(alive), int(k_min)):
        members = ranked[:k]
        value = k * min(float(p[i]) for i in members)
        if best is None or value >= best[3]:            # ties: the larger degree
            best = (k, sorted(members), sorted(set(alive) - set(members)), value)
    return best if best is not None else (0, [], alive, 0.0)
