"""Brute-force definition of the layer-wise strategy plan the search engine must find.

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests may call this module; it shares no code with the
library's search and never imports it.

The paper (section 3, "Dynamic Strategy Selector", discovery phase; section 2, "Layer-Specific
Parallelism Optimization") says that a plan assigns one parallelism strategy to every layer and
that it is found by a dynamic program, driven by a model of each candidate's cost, over a search
space pruned by a decision tree; it prints neither the model nor the recurrence.  The reading taken here is the
plainest problem such a search can be solving:

    given   L layers, S candidate strategies,
            time[l][s]  (ms)    cost of running layer l under strategy s (from the cost table),
            mem[l][s]   (bytes) memory layer l holds on one GPU under strategy s,
            switch[s][s'] (ms)  cost of handing activations from a layer run under s to the next
                                layer run under s' (0 on the diagonal), optional,
            a memory budget B and a memory quantum q (every mem[l][s] is first rounded UP to a
            multiple of q, see round_up; q = 0 leaves them as they are),
    choose  one strategy per layer, c[0..L-1], with  sum_l mem'[l][c_l] <= B,
    minimising  sum_l time[l][c_l] + sum_{l>0} switch[c_{l-1}][c_l].

This module solves it by trying every one of the S^L assignments (tiny L and S only), which is
the definition itself.  Ties in total time are broken towards less memory, then towards the
lexicographically smallest assignment, so that the answer is unique.

Pins (tests/test_oracle_plan.py): with no binding budget and no switch cost the optimum is the
per-layer argmin; with a budget equal to the least possible memory only least-memory strategies
survive; with a prohibitive switch cost the plan is uniform; a hand-worked 3-layer example.
"""
from __future__ import annotations

import itertools
import math
from fractions import Fraction


def round_up(x, q):
    """Memory after rounding (the rule as the library's header states it): k * q for the least whole
    k whose product k * q, formed in double precision, is not below x; q <= 0 leaves x as it is.
    Found here by exact rational division for a starting point one below the quotient's floor and
    a linear search upwards."""
    if q <= 0:
        return x
    k = max(0, math.floor(Fraction(x) / Fraction(q)) - 1)
    while float(k) * q < x:
        k += 1
    return float(k) * q


def plan_cost(choice, time, mem, switch, quantum):
    t = sum(time[l][s] for l, s in enumerate(choice))
    if switch is not None:
        t += sum(switch[a][b] for a, b in zip(choice[:-1], choice[1:]))
    m = sum(round_up(mem[l][s], quantum) for l, s in enumerate(choice))
    return t, m


def brute_force_plan(time, mem, switch, budget, quantum=0.0):
    """Returns (choice tuple, total time, total rounded memory), or None when nothing fits."""
    L = len(time)
    S = len(time[0])
    best = None
    for choice in itertools.product(range(S), repeat=L):
        t, m = plan_cost(choice, time, mem, switch, quantum)
        if m > budget:
            continue
        key = (t, m, choice)
        if best is None or key < best:
            best = key
    if best is None:
        return None
    return best[2], best[0], best[1]
