"""Pins of the interval stage-time oracle and of the stage search over a table of interval times (CPU only).

Sec. 3 gives every pipeline stage its own SPMD plan and Sec. 5.1 balances the stages; on an operator chain the
time of stage [i, j) is then the least value of Sec. 4.2's objective over the plans of operators i..j-1 alone.
The table is checked against the definition (all plans of every interval), a closed form, the chain oracle on
sliced inputs and invariants; the stage search over a table against all cut sets, the additive special case and
closed forms.
"""
import itertools

import numpy as np
import pytest

import oracle

INF = 1 << 52


def all_plans(c, R, i, j):
    """min over x_i..x_{j-1} of sum c[l][x_l] + sum R[l][x_l][x_{l+1}], by enumeration; anything >= INF is INF."""
    K = c.shape[1]
    best = INF
    for x in itertools.product(range(K), repeat=j - i):
        t = 0
        for n, l in enumerate(range(i, j)):
            t += int(c[l, x[n]])
            if l + 1 < j:
                t += int(R[l, x[n], x[n + 1]])
        best = min(best, t)
    return min(best, INF)


def random_chain(rng, L, K, hi_c=50, hi_r=80):
    c = rng.integers(0, hi_c, size=(L, K)).astype(np.int64)
    R = rng.integers(0, hi_r, size=(max(L - 1, 0), K, K)).astype(np.int64)
    return c, R


@pytest.mark.parametrize("seed", range(5))
def test_table_against_all_plans(seed):
    rng = np.random.default_rng(seed)
    L, K = int(rng.integers(1, 6)), int(rng.integers(1, 4))
    c, R = random_chain(rng, L, K, 6 if seed % 2 else 50, 6 if seed % 2 else 80)
    if seed == 3 and L > 1:
        R[0, 0, :] = INF                                  # a producer strategy nobody can consume
    if seed == 4 and L > 2:
        c[1, :] = INF                                     # an operator that cannot run at all
    T = oracle.interval_costs(c, R)
    for i in range(L):
        for j in range(L + 1):
            assert T[i, j] == (all_plans(c, R, i, j) if j > i else INF), (i, j)


def test_one_candidate_and_free_edges_give_prefix_differences():
    rng = np.random.default_rng(10)
    cost = rng.integers(0, 1000, size=37).astype(np.int64)
    T = oracle.interval_costs(cost[:, None].copy(), np.zeros((36, 1, 1), dtype=np.int64))
    P = np.concatenate([[0], np.cumsum(cost)])
    for i in range(37):
        assert np.array_equal(T[i, i + 1:], P[i + 1:] - P[i])
        assert (T[i, :i + 1] == INF).all()


def test_rows_match_the_chain_oracle_on_sliced_inputs_and_padding_is_inert():
    rng = np.random.default_rng(11)
    L, K = 40, 7
    c, R = random_chain(rng, L, K, 10**6, 10**7)
    T = oracle.interval_costs(c, R, ldT=48, nthreads=2)
    assert (T[:, L + 1:] == -1).all()                     # beyond column L nothing is written
    for i, j in [(0, L), (0, 1), (5, 6), (3, 29), (17, 40), (39, 40)]:
        _, _, total, _ = oracle.chain(c[None, i:j].copy(), R[None, i:j - 1].copy())
        assert T[i, j] == total[0]
    # slots padded with INF node costs change nothing
    cp = np.full((L, 16), INF, dtype=np.int64); cp[:, :K] = c
    Rp = rng.integers(0, 5, size=(L - 1, 16, 16)).astype(np.int64); Rp[:, :K, :K] = R
    assert np.array_equal(oracle.interval_costs(cp, Rp)[:, :L + 1], T[:, :L + 1])


def test_longer_stages_cost_more():
    rng = np.random.default_rng(12)
    c, R = random_chain(rng, 30, 5)
    T = oracle.interval_costs(c, R)
    for i in range(30):
        assert (np.diff(T[i, i + 1:]) >= 0).all()         # one more operator at the end never helps
    for j in range(2, 31):
        assert (np.diff(T[:j, j]) <= 0).all()             # dropping the first operator never hurts


def table_cut_sets(T, j, s):
    """min over 0=b0<...<bs=j of max T[b_t][b_{t+1}], by enumeration."""
    best = None
    for cuts in itertools.combinations(range(1, j), s - 1):
        b = (0,) + cuts + (j,)
        m = max(min(int(T[b[t], b[t + 1]]), INF) for t in range(s))
        best = m if best is None or m < best else best
    return best


@pytest.mark.parametrize("seed", range(6))
def test_search_against_all_cut_sets(seed):
    rng = np.random.default_rng(100 + seed)
    L = int(rng.integers(1, 11))
    T = rng.integers(0, 5 if seed % 2 else 1000, size=(L, L + 3)).astype(np.int64)   # any table, not only monotone
    if seed >= 4:
        T[rng.random(T.shape) < 0.3] = INF
    S = L
    bott, cut, _ = oracle.stage_interval(T[None], S)
    dp = {(s, j): table_cut_sets(T, j, s) for s in range(1, S + 1) for j in range(s, L + 1)}
    for s in range(1, S + 1):
        assert bott[0, s - 1] == dp[(s, L)]
        for j in range(L + 1):
            if j < s:
                assert cut[0, s - 1, j] == -1
            elif s == 1:
                assert cut[0, 0, j] == 0
            else:
                want = min(i for i in range(s - 1, j)
                           if max(dp[(s - 1, i)], min(int(T[i, j]), INF)) == dp[(s, j)])
                assert cut[0, s - 1, j] == want


def test_prefix_difference_table_reduces_to_the_additive_search():
    rng = np.random.default_rng(13)
    for L, S, lo in [(60, 9, 1), (33, 33, 0), (128, 16, 0)]:
        cost = rng.integers(lo, 4 if lo == 0 else 500, size=(2, L)).astype(np.int64)   # zero costs: ties
        T = np.full((2, L, L + 1), INF, dtype=np.int64)
        for p in range(2):
            P = np.concatenate([[0], np.cumsum(cost[p])])
            for i in range(L):
                T[p, i, i + 1:] = P[i + 1:] - P[i]
        a = oracle.stage_interval(T, S, s_query=S, nthreads=2)
        b = oracle.stage_dp(cost, S, s_query=S)
        for x, y in zip(a, b):
            assert np.array_equal(x, y)


def test_closed_forms_and_dead_tables():
    rng = np.random.default_rng(14)
    L = 12
    T = rng.integers(1, 100, size=(1, L, L + 1)).astype(np.int64)
    bott, cut, bounds = oracle.stage_interval(T, L, s_query=L)
    assert bott[0, 0] == T[0, 0, L]                                     # one stage: the whole chain
    assert bott[0, L - 1] == max(T[0, i, i + 1] for i in range(L))      # L stages: one operator each
    assert list(bounds[0]) == list(range(L + 1))
    dead = np.full((1, 5, 6), INF, dtype=np.int64)
    bott, cut, bounds = oracle.stage_interval(dead, 3, s_query=3)
    assert (bott == INF).all()
    assert list(cut[0, 2]) == [-1, -1, -1, 2, 2, 2] and list(cut[0, 1]) == [-1, -1, 1, 1, 1, 1]   # lowest i
    assert list(bounds[0]) == [0, 1, 2, 5]


def test_stages_found_on_a_table_of_chain_optima_are_consistent():
    rng = np.random.default_rng(15)
    L, K, S = 50, 6, 7
    c, R = random_chain(rng, L, K, 10**5, 10**5)
    T = oracle.interval_costs(c, R)
    bott, cut, bounds = oracle.stage_interval(T[None], S, s_query=S)
    b = bounds[0]
    assert b[0] == 0 and b[S] == L and (np.diff(b) > 0).all()
    assert bott[0, S - 1] == max(T[b[t], b[t + 1]] for t in range(S))
    assert (np.diff(bott[0]) <= 0).all()                                # more stages never raise the bottleneck
    # the additive search on per-operator minima ignores the edges: it can only be lower
    lower, _, _ = oracle.stage_dp(c.min(axis=1)[None].copy(), S)
    assert (lower[0] <= bott[0]).all()


@pytest.mark.parametrize("seed", range(4))
def test_banded_table_against_all_plans_and_limited_cut_sets(seed):
    # No stage longer than max_len operators (Sec. 5.2 keeps operators near their balanced stage): inside the band
    # the table is the definition, outside it is infeasible, and the search over it is the best cut set among
    # those whose stages all respect the limit, stage times by enumeration of plans.
    rng = np.random.default_rng(200 + seed)
    L, K = int(rng.integers(3, 8)), int(rng.integers(1, 4))
    max_len = int(rng.integers(1, L + 2))                 # from single-operator stages to no limit at all
    c, R = random_chain(rng, L, K, 6 if seed % 2 else 50, 6 if seed % 2 else 80)
    T = oracle.interval_costs(c, R, max_len=max_len)
    for i in range(L):
        for j in range(L + 1):
            want = all_plans(c, R, i, j) if i < j <= i + max_len else INF
            assert T[i, j] == want, (i, j, max_len)
    full = oracle.interval_costs(c, R)
    if max_len >= L:
        assert np.array_equal(T, full)
    S = L
    bott, _, _ = oracle.stage_interval(T[None], S)
    for s in range(1, S + 1):
        best = INF
        for cuts in itertools.combinations(range(1, L), s - 1):
            b = (0,) + cuts + (L,)
            if all(b[t + 1] - b[t] <= max_len for t in range(s)):
                best = min(best, max(all_plans(c, R, b[t], b[t + 1]) for t in range(s)))
        assert bott[0, s - 1] == best, (s, max_len)


def test_banded_table_of_single_operator_stages():
    rng = np.random.default_rng(210)
    c, R = random_chain(rng, 9, 3)
    T = oracle.interval_costs(c, R, max_len=1)
    for i in range(9):
        assert T[i, i + 1] == c[i].min() and (np.delete(T[i, :10], i + 1) == INF).all()
