"""The library's plan search (host code behind the C ABI) against the brute-force oracle on small
problems: total time and memory must agree and the returned assignment must be feasible and
achieve them (several assignments can tie, so the assignment itself is only validated)."""
import os

import numpy as np
import pytest

from oracle import plan as P
from paper_2504_03662_amd import binding as gx


@pytest.fixture(scope="module", autouse=True)
def lib():
    if not os.path.exists(gx.LIB_PATH):
        from paper_2504_03662_amd.build import build
        build(verbose=False)
    return gx.lib()


def _problem(L, S, seed, with_switch, grid=False):
    rng = np.random.default_rng([77, seed])
    if grid:     # few distinct values: many ties
        time = rng.integers(1, 4, (L, S)).astype(float)
        mem = rng.integers(1, 5, (L, S)).astype(float)
    else:
        time = rng.uniform(1.0, 5.0, (L, S))
        mem = rng.uniform(1.0, 9.0, (L, S))
        mem = mem - 0.6 * (time - 1.0)             # faster tends to be heavier, as in the real table
        mem = np.maximum(mem, 0.5)
    sw = None
    if with_switch:
        sw = rng.uniform(0.0, 1.5, (S, S))
        np.fill_diagonal(sw, 0.0)
    return time.tolist(), mem.tolist(), None if sw is None else sw.tolist()


@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("with_switch", [False, True])
@pytest.mark.parametrize("grid", [False, True])
def test_matches_brute_force(seed, with_switch, grid):
    L, S = [(3, 4), (5, 3), (6, 3), (4, 4)][seed % 4]
    time, mem, sw = _problem(L, S, seed, with_switch, grid)
    lo = sum(min(r) for r in mem)
    hi = sum(max(r) for r in mem)
    for frac in (0.0, 0.15, 0.4, 0.7, 1.0):
        for quantum in (0.0, 1.0):
            budget = lo + frac * (hi - lo) + (0.0 if quantum == 0.0 else L * quantum * 0.5)
            ref = P.brute_force_plan(time, mem, sw, budget, quantum)
            st, choice, res = gx.plan_search(time, mem, sw, budget=budget, quantum=quantum, check=False)
            if ref is None:
                assert st == 9
                continue
            assert st == gx.GX_OK
            t, m = P.plan_cost(choice, time, mem, sw, quantum)
            assert m <= budget + 1e-9
            assert abs(t - res.total_ms) < 1e-9 and abs(m - res.total_mem_bytes) < 1e-9
            assert abs(res.total_ms - ref[1]) < 1e-9, (choice, ref)
            assert abs(res.total_mem_bytes - ref[2]) < 1e-9, (choice, ref)


def test_infeasible_and_argument_errors():
    time, mem, sw = _problem(3, 3, 1, True)
    st, _, _ = gx.plan_search(time, mem, sw, budget=0.1, check=False)
    assert st == 9 and "budget" in gx.status_str(9)
    bad = [row[:] for row in time]
    bad[1][1] = float("nan")
    assert gx.plan_search(bad, mem, sw, budget=100.0, check=False)[0] == 2
    neg = [row[:] for row in mem]
    neg[0][0] = -1.0
    assert gx.plan_search(time, neg, sw, budget=100.0, check=False)[0] == 2
    assert gx.plan_search(time, mem, sw, budget=-1.0, check=False)[0] == 2
    import ctypes
    prob = gx.PlanProblem(0, 3, None, None, None, 1.0, 0.0)
    res = gx.PlanResult()
    c = (ctypes.c_int32 * 3)()
    assert gx.lib().gx_plan_search(ctypes.byref(prob), c, ctypes.byref(res)) == 1      # NULL tables
    assert gx.lib().gx_plan_search(None, c, ctypes.byref(res)) == 1


def test_model_sized_problem_is_consistent():
    """48 layers, 12 strategies, identical layers: the plan must fit, must not lose against any
    uniform plan or the greedy per-layer choice under the budget, and must use the budget well."""
    rng = np.random.default_rng(5)
    S, L = 12, 48
    t_row = np.sort(rng.uniform(2.0, 9.0, S))
    m_row = np.sort(rng.uniform(1.0, 12.0, S))[::-1].copy()       # faster = heavier
    time = [t_row.tolist()] * L
    mem = [m_row.tolist()] * L
    sw = (0.3 * np.abs(np.subtract.outer(np.arange(S), np.arange(S)))).tolist()
    budget = 0.5 * (m_row.min() + m_row.max()) * L
    st, choice, res = gx.plan_search(time, mem, sw, budget=budget, quantum=0.05)
    t, m = P.plan_cost(choice, time, mem, sw, 0.05)
    assert m <= budget and abs(t - res.total_ms) < 1e-9
    for s in range(S):
        tu, mu = P.plan_cost([s] * L, time, mem, sw, 0.05)
        if mu <= budget:
            assert res.total_ms <= tu + 1e-9
    assert res.total_ms < P.plan_cost([S - 1] * L, time, mem, sw, 0.05)[0]   # better than all-lightest
    assert res.frontier_peak >= 1 and res.pruned >= 0
    # without switching costs dominated strategies are pruned and the optimum only improves
    st2, choice2, res2 = gx.plan_search(time, mem, None, budget=budget, quantum=0.05)
    assert res2.total_ms <= res.total_ms + 1e-9


def test_quantum_rounding_rule_through_the_abi():
    """The library's own rounding, observed as the total memory of a one-layer, one-strategy plan,
    against values worked out by hand from the rule in the header (least whole k with
    k * q >= x in double arithmetic): exact multiples stay, one unit in the last place above moves
    to the next multiple, one below stays."""
    def rounded(x, q):
        st, choice, res = gx.plan_search([[1.0]], [[x]], None, budget=1e300, quantum=q, check=False)
        assert st == gx.GX_OK and choice == [0]
        return res.total_mem_bytes

    for q in (4.0, 3.0, 1024.0, 0.1, 1e9 / 7):
        for k in (1, 2, 3, 7, 1000):
            m = float(k) * q
            assert rounded(m, q) == m
            assert rounded(float(np.nextafter(m, np.inf)), q) == float(k + 1) * q
            assert rounded(float(np.nextafter(m, -np.inf)), q) == m
    assert rounded(5.0, 0.0) == 5.0 and rounded(5.0, 4.0) == 8.0 and rounded(0.0, 4.0) == 0.0
    assert rounded(0.3, 0.1) == 3 * 0.1 and rounded(float(np.nextafter(3 * 0.1, 1.0)), 0.1) == 4 * 0.1


def test_single_layer_reports_its_frontier():
    st, choice, res = gx.plan_search([[2.0, 1.0]], [[1.0, 2.0]], None, budget=10.0, check=False)
    assert st == gx.GX_OK and choice == [1] and res.frontier_peak == 1
