"""Pins for the brute-force plan oracle: special cases whose answer is known without any search."""
import numpy as np

from oracle import plan as P


def _rand(L, S, seed):
    rng = np.random.default_rng(seed)
    time = rng.uniform(1.0, 5.0, (L, S)).tolist()
    mem = rng.uniform(1.0, 9.0, (L, S)).tolist()
    sw = rng.uniform(0.1, 1.0, (S, S))
    np.fill_diagonal(sw, 0.0)
    return time, mem, sw.tolist()


def test_unconstrained_without_switch_cost_is_per_layer_argmin():
    time, mem, _ = _rand(5, 3, 1)
    choice, t, m = P.brute_force_plan(time, mem, None, budget=1e9)
    assert list(choice) == [int(np.argmin(row)) for row in time]
    assert abs(t - sum(min(row) for row in time)) < 1e-12


def test_tight_budget_forces_least_memory():
    time, mem, sw = _rand(4, 3, 2)
    least = sum(min(row) for row in mem)
    choice, t, m = P.brute_force_plan(time, mem, sw, budget=least * (1 + 1e-12))
    assert list(choice) == [int(np.argmin(row)) for row in mem]
    assert P.brute_force_plan(time, mem, sw, budget=least * 0.999) is None


def test_prohibitive_switch_cost_gives_a_uniform_plan():
    time, mem, _ = _rand(5, 3, 3)
    S = 3
    sw = [[0.0 if a == b else 1e6 for b in range(S)] for a in range(S)]
    choice, t, m = P.brute_force_plan(time, mem, sw, budget=1e9)
    assert len(set(choice)) == 1
    col = int(np.argmin(np.sum(np.array(time), axis=0)))
    assert choice[0] == col and abs(t - np.sum(np.array(time)[:, col])) < 1e-12


def test_hand_worked_example():
    # two strategies: 0 = fast but heavy (2 ms, 6 units), 1 = slow but light (3 ms, 2 units);
    # three layers, budget 12 units, switching costs 0.4 ms.
    # all fast = 18 units (no); two fast = 14 (no); one fast + two slow = 10 units (fits), 8 ms + switches:
    # fast at an end -> one switch (8.4 ms), fast in the middle -> two (8.8 ms); all slow = 9 ms.
    time = [[2.0, 3.0]] * 3
    mem = [[6.0, 2.0]] * 3
    sw = [[0.0, 0.4], [0.4, 0.0]]
    choice, t, m = P.brute_force_plan(time, mem, sw, budget=12.0)
    assert choice == (0, 1, 1) and abs(t - 8.4) < 1e-12 and m == 10.0      # ties broken lexicographically
    # a quantum of 4 rounds the light layers up to 4 units: 6 + 4 + 4 = 14 no longer fits, all slow does
    choice, t, m = P.brute_force_plan(time, mem, sw, budget=12.0, quantum=4.0)
    assert choice == (1, 1, 1) and abs(t - 9.0) < 1e-12 and m == 12.0


def test_round_up_rule_on_exact_multiples_and_their_one_ulp_neighbours():
    # hand-worked from the stated rule: least whole k with k * q (in double) >= x
    assert P.round_up(5.0, 0) == 5.0 and P.round_up(5.0, 4.0) == 8.0
    for q in (4.0, 3.0, 1024.0, 0.1, 1e9 / 7):
        for k in (1, 2, 3, 7, 1000):
            m = float(k) * q                                   # a multiple, as formed in double precision
            assert P.round_up(m, q) == m                       # stays
            assert P.round_up(np.nextafter(m, np.inf), q) == float(k + 1) * q      # one ulp above: next multiple
            assert P.round_up(np.nextafter(m, -np.inf), q) == m                    # one ulp below: this multiple
    assert P.round_up(0.0, 4.0) == 0.0 and P.round_up(1e-300, 4.0) == 4.0
    # the decimal 0.3 lies below the double product 3 * 0.1 = 0.30000000000000004, which lies below 4 * 0.1
    assert P.round_up(0.3, 0.1) == 3 * 0.1 and P.round_up(3 * 0.1, 0.1) == 3 * 0.1
    assert P.round_up(np.nextafter(3 * 0.1, 1.0), 0.1) == 4 * 0.1


# pipeline regrouping (oracle/regroup.py) ---------------------------------------------------------

def test_regroup_closed_forms():
    from oracle import regroup as R
    ms = [3.0, 1.0, 4.0, 1.0, 5.0, 9.0, 2.0, 6.0]
    assert R.best_bottleneck(ms, 1)[0] == sum(ms)
    assert R.best_bottleneck(ms, len(ms))[0] == max(ms)
    for L in range(1, 9):
        for P in range(1, L + 1):
            assert R.best_bottleneck([2.5] * L, P)[0] == 2.5 * -(-L // P)


def test_regroup_bounds_and_monotonicity():
    import random
    from oracle import regroup as R
    rng = random.Random(7)
    for _ in range(40):
        L = rng.randint(1, 9)
        ms = [rng.choice([0.5, 1.0, 1.5, 2.0, 7.0]) for _ in range(L)]
        prev = None
        for P in range(1, L + 1):
            b, first = R.best_bottleneck(ms, P)
            assert R.is_grouping(first, L, P) and R.bottleneck(ms, first) == b
            lower = max(max(ms), sum(ms) / P)
            assert lower <= b <= lower + max(ms)
            assert prev is None or b <= prev
            prev = b


def test_regroup_hand_worked():
    from oracle import regroup as R
    # 1 2 3 4 5 in two stages: {1 2 3 | 4 5} gives max(6, 9) = 9, {1 2 3 4 | 5} gives 10, {1 2 | 3 4 5} 12
    assert R.best_bottleneck([1.0, 2.0, 3.0, 4.0, 5.0], 2) == (9.0, (0, 3, 5))
    # in three: {1 2 3 | 4 | 5} -> 6
    assert R.best_bottleneck([1.0, 2.0, 3.0, 4.0, 5.0], 3) == (6.0, (0, 3, 4, 5))
    # six layers from stages {0 1 | 2 3 | 4 5} to {0 1 2 | 3 4 5}: layer 2 goes from stage 1 to 0,
    # layers 4 and 5 from stage 2 to 1; layer 3 stays in stage 1, layers 0 and 1 in stage 0
    assert R.moves(6, (0, 2, 4, 6), (0, 3, 6)) == ([0, 0, 0, 1, 1, 1], 3)
    assert R.moves(4, (0, 4), (0, 1, 2, 3, 4)) == ([0, 1, 2, 3], 3)
