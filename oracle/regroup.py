"""Brute-force definition of the pipeline regrouping the library must find.

TEST INFRASTRUCTURE, NOT PRODUCT CODE.  Only tests may call this module; it shares no code with the
library and never imports it.

The paper (section 4, "Handling Transitions") says that a pipeline-parallel transition changes how
layers are grouped and that every process is then told which layers to hold; it gives no rule for
the grouping.  The reading taken here: a stage holds consecutive layers, every stage at least one,
and a grouping is as good as its slowest stage,

    bottleneck(first) = max over stages s of  sum of layer_ms[first[s] .. first[s+1]-1],

so the grouping wanted is one that minimises the bottleneck.  Several groupings can reach the
minimum; what is unique is the minimum itself, so the tests compare that and check that the
library's grouping is a grouping and reaches it.

This module tries every way of cutting L layers into P consecutive non-empty groups (tiny L only),
which is the definition itself, and counts moved layers by looking each layer up in both groupings.

Pins (tests/test_oracle_plan.py): one stage is the total and as many stages as layers is the largest
layer; equal layers give ceil(L / P) layers' time; the result is never below max(largest layer,
total / P) and never above it by more than the largest layer; one more stage never makes it worse;
a hand-worked case; moves counted by hand.
"""
from __future__ import annotations

import itertools


def bottleneck(layer_ms, first):
    return max(sum(layer_ms[first[s]:first[s + 1]]) for s in range(len(first) - 1))


def is_grouping(first, layers, stages):
    return (len(first) == stages + 1 and first[0] == 0 and first[-1] == layers
            and all(first[s] < first[s + 1] for s in range(stages)))


def best_bottleneck(layer_ms, stages):
    """Smallest bottleneck over all groupings, and one grouping that reaches it."""
    L = len(layer_ms)
    best = None
    for cuts in itertools.combinations(range(1, L), stages - 1):
        first = (0,) + cuts + (L,)
        b = bottleneck(layer_ms, first)
        if best is None or b < best[0]:
            best = (b, first)
    return best


def stage_of(first, layer):
    for s in range(len(first) - 1):
        if first[s] <= layer < first[s + 1]:
            return s
    raise ValueError("layer outside the grouping")


def moves(layers, old_first, new_first):
    """(stage of every layer afterwards, number of layers whose stage index changes)."""
    new = [stage_of(new_first, l) for l in range(layers)]
    moved = sum(1 for l in range(layers) if stage_of(old_first, l) != new[l])
    return new, moved
