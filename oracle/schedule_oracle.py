"""Execution order of offloaded experts and the timeline it produces.

TEST INFRASTRUCTURE ONLY.  Nothing on the product path may import this module; it shares no code
with the library's host scheduler.

What it states (CPM-2 paper, arxiv 2106.10715, Section 6.2, the part on scheduling offloaded experts):

* expert i needs alpha_i seconds of computation (its floating-point operations over the peak rate,
  proportional to its token count) and every expert needs the same beta seconds of parameter
  loading (parameter bytes over the peak transfer rate); at most K experts are resident at a time;
* loading and computing run on different streams, an expert's load must precede its computation;
* the computation order o_1..o_T should satisfy, for every 1 <= t <= T,
      sum_{i<t} alpha_{o_i} >= (t - 1) beta          (each load is covered by earlier computation)
      sum_{i<t} alpha_{o_i} <= (t + K - 1) beta      (never more than K experts resident)
  and is produced by "a greedy algorithm"; the constraints may be unsatisfiable.

The paper does not print the greedy rule.  Reading used here: walk the positions in order and keep
the slack S = sum of chosen alpha - (chosen count) * beta; at every position take the remaining
expert with the largest alpha whose choice keeps S <= K beta (heavy experts early build the slack
that light ones consume), and if no remaining expert keeps it, the one with the smallest alpha.
Ties go to the lower expert index.  The order is reported together with whether it satisfies both
constraints.  When every alpha is below beta (loading dominates, the usual case at small batch),
this degenerates to "most tokens first", which puts the shortest computation after the last load.

timeline() is the plain two-engine model those constraints are derived from: one copy engine, one
compute engine, K slots, loads in execution order, a slot is reused once its expert has finished.
"""
from __future__ import annotations

from typing import List, NamedTuple, Sequence, Tuple


class Timeline(NamedTuple):
    load_start: List[float]
    load_end: List[float]
    comp_start: List[float]
    comp_end: List[float]
    makespan: float
    compute_wait: float      # time the compute engine idles waiting for a load, after the first load


def timeline(alpha_in_order: Sequence[float], beta: float, K: int) -> Timeline:
    """Discrete-event run of experts in the given order (Section 6.2, Figure 4)."""
    if K < 1:
        raise ValueError("K must be at least 1")
    n = len(alpha_in_order)
    ls, le, cs, ce = [0.0] * n, [0.0] * n, [0.0] * n, [0.0] * n
    wait = 0.0
    for t in range(n):
        copy_free = le[t - 1] if t > 0 else 0.0
        slot_free = ce[t - K] if t >= K else 0.0           # the slot of the expert K positions earlier
        ls[t] = max(copy_free, slot_free)
        le[t] = ls[t] + beta
        compute_free = ce[t - 1] if t > 0 else 0.0
        cs[t] = max(compute_free, le[t])
        if t > 0:
            wait += cs[t] - compute_free
        ce[t] = cs[t] + alpha_in_order[t]
    return Timeline(ls, le, cs, ce, ce[-1] if n else 0.0, wait)


def constraints_hold(alpha_in_order: Sequence[float], beta: float, K: int) -> Tuple[bool, bool]:
    """(first constraint holds for all t, second constraint holds for all t), Section 6.2."""
    covered, bounded = True, True
    prefix = 0.0
    for t in range(1, len(alpha_in_order) + 1):
        if prefix < (t - 1) * beta:
            covered = False
        if prefix > (t + K - 1) * beta:
            bounded = False
        prefix += alpha_in_order[t - 1]
    return covered, bounded


def greedy_order(alpha: Sequence[float], beta: float, K: int) -> Tuple[List[int], bool]:
    """Order of the experts 0..len(alpha)-1 by the greedy reading above, and whether it satisfies both
    constraints."""
    remaining = list(range(len(alpha)))
    order: List[int] = []
    chosen_sum = 0.0
    while remaining:
        placed = len(order)
        fits = [i for i in remaining if chosen_sum + alpha[i] - (placed + 1) * beta <= K * beta]
        if fits:
            pick = max(fits, key=lambda i: (alpha[i], -i))
        else:
            pick = min(remaining, key=lambda i: (alpha[i], i))
        order.append(pick)
        remaining.remove(pick)
        chosen_sum += alpha[pick]
    covered, bounded = constraints_hold([alpha[i] for i in order], beta, K)
    return order, covered and bounded


# ---------------------------------------------------------------------------------- resident experts
#
# Section 6.2: "only the parameters of a certain number (denoted as K ...) of experts can reside in GPU
# memory simultaneously".  When K slots outlive a call, an expert that is still resident need not be
# loaded again.  Which resident expert gives way when a slot is needed is not the paper's subject; the
# reading used here: the whole execution order of a call is known before its first load, so the expert
# whose next use in this call lies furthest ahead goes (never used again = furthest of all; among those
# the one unused for longest, then the lowest slot) - the classical optimal replacement for a known
# request sequence, which minimises the loads of the call.

def plan_slots(order: Sequence[int], slot_expert: Sequence[int], slot_tick: Sequence[int], tick: int):
    """For each position of `order`: (slot, load?) given the experts the K slots hold (-1 = empty) and when
    each slot was last used.  Returns (slots, loads, slot_expert_after, slot_tick_after, tick_after)."""
    held = list(slot_expert)
    used = list(slot_tick)
    slots, loads = [], []
    for pos, e in enumerate(order):
        if e in held:
            s = held.index(e)
            loads.append(False)
        else:
            def next_use(x):
                for j in range(pos + 1, len(order)):
                    if order[j] == x:
                        return j
                return len(order) + 1                      # never again in this call
            # empty slots first, then furthest next use, then least recently used, then lowest slot
            s = min(range(len(held)),
                    key=lambda i: (0 if held[i] < 0 else 1, -(next_use(held[i]) if held[i] >= 0 else 0), used[i], i))
            held[s] = e
            loads.append(True)
        tick += 1
        used[s] = tick
        slots.append(s)
    return slots, loads, held, used, tick
