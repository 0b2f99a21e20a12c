"""Pins of the chain-DP oracle (CPU only).

Nothing here calls the GPU library.  The oracle is checked against things it
does not contain: exhaustive evaluation of the objective C of Sec. 4.2 over
all K^N plans, a library shortest-path routine on the layered graph, closed
forms and invariances.
"""
import itertools

import numpy as np
import pytest
import scipy.sparse as sp
from scipy.sparse.csgraph import shortest_path

import oracle
from paper_2302_08141_amd.workloads import synthetic as syn

INF = oracle.INF


def brute_force(c, R):
    """Evaluate C(x) = sum c_i[x_i] + sum R_i[x_i][x_{i+1}] for every plan x.

    Returns (minimum, the optimal plan that is smallest when compared from the
    LAST operator backwards) -- the plan a forward sweep with lowest-index ties
    and a backward walk must return.
    """
    N, K = c.shape
    plans = np.array(list(itertools.product(range(K), repeat=N)), dtype=np.int64)  # [K^N][N]
    cost = np.zeros(len(plans), dtype=np.int64)
    for i in range(N):
        cost += c[i, plans[:, i]]
    for i in range(N - 1):
        cost += R[i, plans[:, i], plans[:, i + 1]]
    cost = np.minimum(cost, INF)       # any infeasible term makes the plan infeasible
    best = cost.min()
    cand = plans[cost == best]
    key = np.zeros(len(cand), dtype=np.int64)
    for i in range(N - 1, -1, -1):     # x_{N-1} most significant
        key = key * K + cand[:, i]
    return int(best), cand[np.argmin(key)].astype(np.int32)


def run_oracle(c, R):
    arg, vfinal, total, last = oracle.chain(np.ascontiguousarray(c[None]), np.ascontiguousarray(R[None]))
    plan = oracle.backtrack(arg, last)
    return int(total[0]), plan[0], arg[0], vfinal[0], int(last[0])


def test_tiny_chain_config_all_plans():
    # N=10, K=4: 4^10 = 1,048,576 plans
    w = syn.TINY_CHAIN
    c, R = syn.random_chain_problem(0, w["N"], w["K"], w["c_range"], w["r_range"])
    assert c.min() >= 0 and c.max() < 1000 and R.max() < 5000
    assert all(R[i, a, a] == 0 for i in range(9) for a in range(4))
    best, plan = brute_force(c, R)
    total, oplan, *_ = run_oracle(c, R)
    assert total == best
    assert np.array_equal(oplan, plan)
    assert oracle.plan_cost(np.ascontiguousarray(c), np.ascontiguousarray(R), oplan) == best


@pytest.mark.parametrize("seed", range(12))
def test_random_tiny_with_ties_ragged_and_infeasible(seed):
    rng = np.random.default_rng(1000 + seed)
    N = int(rng.integers(1, 8))
    K = int(rng.integers(1, 6))
    lo_hi = (0, 3) if seed % 2 == 0 else (0, 50)     # {0,1,2} forces many ties
    c = rng.integers(*lo_hi, size=(N, K)).astype(np.int64)
    R = rng.integers(*lo_hi, size=(max(N - 1, 0), K, K)).astype(np.int64)
    # ragged candidate counts: slots >= K_i are empty
    Ki = rng.integers(1, K + 1, size=N)
    for i in range(N):
        c[i, Ki[i]:] = INF
        if i < N - 1:
            R[i, Ki[i]:, :] = INF
        if i > 0:
            R[i - 1, :, Ki[i]:] = INF
    # sprinkle infeasible entries
    if seed % 3 == 0 and N > 1:
        mask = rng.random(R.shape) < 0.3
        R[mask] = INF
    if seed == 9:
        c[N // 2, :] = INF                            # nothing feasible at all
    best, plan = brute_force(c, R)
    total, oplan, *_ = run_oracle(c, R)
    assert total == best
    assert np.array_equal(oplan, plan)
    if seed == 9:
        assert total == INF and not oplan.any()


@pytest.mark.parametrize("N,K", [(2, 3), (6, 7), (15, 5)])
def test_total_equals_library_shortest_path(N, K):
    c, R = syn.random_chain_problem(7, N, K, 1000, 5000)
    # layered DAG: source -> (0,j) weight c0[j]; (i,a)->(i+1,b) weight R_i[a][b] + c_{i+1}[b];
    # (N-1,j) -> sink.  Every weight is shifted by +1 so that no edge has weight 0; a
    # source-sink path has exactly N+1 edges.
    nid = lambda i, j: 1 + i * K + j
    sink = 1 + N * K
    rows, cols, w = [], [], []
    for j in range(K):
        rows.append(0); cols.append(nid(0, j)); w.append(c[0, j] + 1)
        rows.append(nid(N - 1, j)); cols.append(sink); w.append(1)
    for i in range(N - 1):
        for a in range(K):
            for b in range(K):
                rows.append(nid(i, a)); cols.append(nid(i + 1, b)); w.append(R[i, a, b] + c[i + 1, b] + 1)
    g = sp.csr_matrix((np.array(w, dtype=np.float64), (rows, cols)), shape=(sink + 1, sink + 1))
    d = shortest_path(g, method="D", directed=True, indices=0)
    total, *_ = run_oracle(c, R)
    assert total == int(round(d[sink])) - (N + 1)


def test_closed_forms():
    N, K = 9, 6
    c, R = syn.random_chain_problem(3, N, K, 1000, 5000)
    # no edge cost: every operator picks its own cheapest candidate (lowest index on ties)
    total, plan, *_ = run_oracle(c, np.zeros_like(R))
    assert total == c.min(axis=1).sum()
    assert np.array_equal(plan, c.argmin(axis=1))
    # one candidate: the only plan
    c1, R1 = c[:, :1].copy(), R[:, :1, :1].copy() + 5
    total, plan, *_ = run_oracle(c1, R1)
    assert total == c1.sum() + R1.sum() and not plan.any()
    # zero diagonal and prohibitive off-diagonal: the constant plan with the best column sum
    big = int(c.max(axis=1).sum()) + 1
    Rb = np.full_like(R, big)
    d = np.arange(K)
    Rb[:, d, d] = 0
    total, plan, *_ = run_oracle(c, Rb)
    j = int(c.sum(axis=0).argmin())
    assert total == c[:, j].sum() and np.all(plan == j)


def test_invariances():
    N, K = 11, 5
    c, R = syn.random_chain_problem(5, N, K, 1000, 5000)
    total, plan, arg, vfinal, last = run_oracle(c, R)
    # adding delta_i to every candidate of operator i shifts the total, not the plan
    delta = np.arange(N, dtype=np.int64) * 17 + 3
    t2, p2, *_ = run_oracle(c + delta[:, None], R)
    assert t2 == total + delta.sum() and np.array_equal(p2, plan)
    # reversing the chain (edge tables transposed) keeps the total
    t3, *_ = run_oracle(c[::-1].copy(), np.ascontiguousarray(R[::-1].transpose(0, 2, 1)))
    assert t3 == total
    # splitting at operator s and joining the two halves over its candidates keeps the total
    for s in (1, 4, N - 2):
        _, _, _, v_left, _ = run_oracle(c[: s + 1].copy(), R[:s].copy())
        cr = c[s:][::-1].copy()
        cr[-1] = 0                                     # operator s is counted on the left
        _, _, _, v_right, _ = run_oracle(cr, np.ascontiguousarray(R[s:][::-1].transpose(0, 2, 1)))
        assert int((v_left + v_right).min()) == total
    # vfinal is what the recurrence says at the last operator
    assert vfinal.min() == total and int(vfinal.argmin()) == last


def test_arg_is_lowest_minimiser_and_plan_cost_matches():
    N, K = 8, 6
    rng = np.random.default_rng(5)
    c = rng.integers(0, 3, size=(N, K)).astype(np.int64)
    R = rng.integers(0, 3, size=(N - 1, K, K)).astype(np.int64)
    total, plan, arg, vfinal, last = run_oracle(c, R)
    v = c[0].copy()
    for i in range(N - 1):
        t = v[:, None] + R[i]                          # [a][b]
        assert np.array_equal(arg[i], t.argmin(axis=0))    # numpy argmin = first minimiser
        v = c[i + 1] + t.min(axis=0)
    assert np.array_equal(v, vfinal)
    assert oracle.plan_cost(c, R, plan) == total


def test_batched_and_shared_R_agree_with_single():
    B, N, K, Kp = 5, 6, 5, 8
    c, R = syn.random_chain_batch(range(B), N, K, 1000, 5000, Kp=Kp)
    arg, vfinal, total, last = oracle.chain(c, R, nthreads=3)
    for p in range(B):
        t, plan, a, vf, l = run_oracle(c[p], R[p])
        assert t == total[p] and l == last[p] and np.array_equal(a, arg[p])
        assert l < K and np.all(plan < K)
    arg_s, _, total_s, _ = oracle.chain(c, np.ascontiguousarray(R[0]), shared_R=True)
    for p in range(B):
        t, *_ = run_oracle(c[p], R[0])
        assert t == total_s[p]


def test_generator_is_splitmix64():
    # first outputs of SplitMix64 seeded with 1234567 (reference values of the published generator)
    s = np.uint64(1234567)
    with np.errstate(over="ignore"):
        got = [int(syn.mix64(s + np.uint64(n + 1) * syn.GOLDEN)) for n in range(3)]
    assert got == [6457827717110365317, 3203168211198807973, 9817491932198370423]
