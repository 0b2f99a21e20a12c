"""Pins of the pipeline-stage oracle (CPU only).

The paper asks for balanced stages (Sec. 2.1; Sec. 5.2: time_per_stage =
sum(comp)/d) and stage ids that never decrease along an edge (Sec. 5.1).  On a
chain that is: choose cut points, minimise the largest stage sum.  The oracle's
recurrence is checked against the definition (all cut sets), a textbook
binary-search + greedy solver, closed forms and invariants.
"""
import itertools

import numpy as np
import pytest

import oracle
from paper_2302_08141_amd.workloads import synthetic as syn


def all_cut_sets(cost, s):
    """min over 0=b0<b1<...<bs=L of the max stage sum, by enumeration."""
    L = len(cost)
    P = np.concatenate([[0], np.cumsum(cost)])
    best = None
    for cuts in itertools.combinations(range(1, L), s - 1):
        b = (0,) + cuts + (L,)
        m = max(P[b[t + 1]] - P[b[t]] for t in range(s))
        best = m if best is None or m < best else best
    return int(best)


def greedy_feasible(cost, s, cap):
    stages, run = 1, 0
    for x in cost:
        if x > cap:
            return False
        if run + x > cap:
            stages += 1
            run = x
        else:
            run += x
    return stages <= s


def linear_partition(cost, s):
    """Smallest cap for which a greedy sweep needs at most s stages (integers, exact)."""
    lo, hi = int(max(cost)), int(sum(cost))
    while lo < hi:
        mid = (lo + hi) // 2
        if greedy_feasible(cost, s, mid):
            hi = mid
        else:
            lo = mid + 1
    return lo


@pytest.mark.parametrize("seed", range(6))
def test_against_all_cut_sets(seed):
    rng = np.random.default_rng(seed)
    L = int(rng.integers(1, 13))
    hi = 4 if seed % 2 else 100                 # small range: many ties
    cost = rng.integers(1, hi, size=L).astype(np.int64)
    S = L
    bott, cut, _ = oracle.stage_dp(cost[None], S)
    P = np.concatenate([[0], np.cumsum(cost)])
    # dp[s][j] for every prefix j, from the definition
    dp = {(s, j): all_cut_sets(cost[:j], s) for s in range(1, S + 1) for j in range(s, L + 1)}
    for s in range(1, S + 1):
        assert bott[0, s - 1] == dp[(s, L)]
        for j in range(L + 1):
            if j < s:
                assert cut[0, s - 1, j] == -1
            elif s == 1:
                assert cut[0, 0, j] == 0
            else:
                # lowest i whose split reaches the optimum
                want = min(i for i in range(s - 1, j)
                           if max(dp[(s - 1, i)], P[j] - P[i]) == dp[(s, j)])
                assert cut[0, s - 1, j] == want


@pytest.mark.parametrize("L,S", [(50, 7), (257, 16), (1000, 64)])
def test_against_binary_search_greedy(L, S):
    cost = syn.segment_costs(L, L)              # [1, 1e5)
    assert cost.min() >= 1 and cost.max() < 100000
    bott, cut, _ = oracle.stage_dp(cost[None], S)
    for s in (1, 2, 3, S // 2, S):
        assert bott[0, s - 1] == linear_partition(cost, s)


def test_closed_forms_and_invariants():
    L, S = 96, 96
    cost = syn.segment_costs(1, L)
    bott, cut, _ = oracle.stage_dp(cost[None], S)
    assert bott[0, 0] == cost.sum()             # one stage holds everything
    assert bott[0, L - 1] == cost.max()         # one segment per stage
    assert np.all(np.diff(bott[0]) <= 0)        # more stages never hurt
    for s in range(1, S + 1):
        lower = max(int(cost.max()), -(-int(cost.sum()) // s))   # ceil(sum/s): perfect balance
        assert bott[0, s - 1] >= lower
    eq = np.full(40, 9, dtype=np.int64)
    b2, _, _ = oracle.stage_dp(eq[None], 40)
    for s in range(1, 41):
        assert b2[0, s - 1] == -(-40 // s) * 9


@pytest.mark.parametrize("s_query", [1, 2, 5, 16])
def test_bounds_reach_the_bottleneck(s_query):
    B, L, S = 3, 200, 16
    cost = np.stack([syn.segment_costs(p, L) for p in range(B)])
    bott, cut, bounds = oracle.stage_dp(cost, S, s_query=s_query, nthreads=2)
    for p in range(B):
        b = bounds[p]
        assert b[0] == 0 and b[-1] == L and np.all(np.diff(b) >= 1)   # stage ids never decrease
        P = np.concatenate([[0], np.cumsum(cost[p])])
        assert max(P[b[t + 1]] - P[b[t]] for t in range(s_query)) == bott[p, s_query - 1]
