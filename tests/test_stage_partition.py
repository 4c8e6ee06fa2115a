"""gx_stage_partition / gx_stage_moves (host code of the library) against oracle/regroup.py: the
smallest bottleneck is unique and is compared exactly up to rounding; the grouping itself may be
any that reaches it, so it is checked for being a grouping, for reaching it, and for the library's
stated choice among equals (every stage, from the first, as short as it can be)."""
import os
import random

import pytest

from oracle import regroup as R
from paper_2504_03662_amd import binding as gx

GX_ERR_SHAPE = 2


@pytest.fixture(scope="module", autouse=True)
def lib():
    if not os.path.exists(gx.LIB_PATH):
        from paper_2504_03662_amd.build import build
        build(verbose=False)
    return gx.lib()


def _shortest_first(ms, stages, opt):
    """The grouping the header promises, found by trying cuts in increasing order (plain search)."""
    L = len(ms)
    first = [0]
    for s in range(stages - 1):
        rest = stages - s - 1
        e = first[-1] + 1
        while True:
            head = sum(ms[first[-1]:e])
            tail = R.best_bottleneck(ms[e:], rest)[0] if L - e >= rest else float("inf")
            if head <= opt * (1 + 1e-12) and tail <= opt * (1 + 1e-12):
                break
            e += 1
        first.append(e)
    return first + [L]


def test_matches_the_brute_force_on_random_small_cases():
    rng = random.Random(11)
    for _ in range(200):
        L = rng.randint(1, 10)
        P = rng.randint(1, L)
        ms = [rng.choice([0.25, 1.0, 1.5, 3.0, 8.0]) * rng.choice([1.0, 1.0, 1.125]) for _ in range(L)]
        want, _ = R.best_bottleneck(ms, P)
        st, first, got = gx.stage_partition(L, P, ms)
        assert st == gx.GX_OK
        assert R.is_grouping(first, L, P)
        assert abs(got - want) <= 1e-12 * want
        assert abs(R.bottleneck(ms, first) - want) <= 1e-12 * want
        assert first == _shortest_first(ms, P, want)


def test_equal_times_when_no_times_are_given():
    for L, P in ((8, 4), (7, 3), (5, 5), (32, 8), (33, 8)):
        st, first, got = gx.stage_partition(L, P, None)
        assert st == gx.GX_OK and R.is_grouping(first, L, P)
        assert got == float(-(-L // P))
        assert max(first[s + 1] - first[s] for s in range(P)) == -(-L // P)


def test_moves_match_the_oracle():
    rng = random.Random(5)
    for _ in range(100):
        L = rng.randint(1, 12)

        def grouping():
            P = rng.randint(1, L)
            return [0] + sorted(rng.sample(range(1, L), P - 1)) + [L]
        old, new = grouping(), grouping()
        st, stage, moved = gx.stage_moves(L, old, new)
        assert st == gx.GX_OK
        assert (stage, moved) == R.moves(L, old, new)


def test_errors():
    assert gx.stage_partition(4, 5, None, check=False)[0] == GX_ERR_SHAPE
    assert gx.stage_partition(0, 1, None, check=False)[0] == GX_ERR_SHAPE
    assert gx.stage_partition(3, 2, [1.0, 0.0, 2.0], check=False)[0] == GX_ERR_SHAPE
    assert gx.stage_partition(3, 2, [1.0, float("nan"), 2.0], check=False)[0] == GX_ERR_SHAPE
    assert gx.stage_moves(4, [0, 2, 4], [0, 3, 3, 4], check=False)[0] == GX_ERR_SHAPE
    assert gx.stage_moves(4, [0, 2, 5], [0, 4], check=False)[0] == GX_ERR_SHAPE
