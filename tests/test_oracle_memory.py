"""Pins of the memory-constrained search oracle (CPU only).

Sec. 4.4: rank parameters by size, forbid replication of the k largest, take
the smallest k whose best plan fits the memory limit.  Checked against
exhaustive search over all plans on tiny chains, and against the plain chain
oracle for k = 0.
"""
import itertools

import numpy as np
import pytest

import oracle

INF = oracle.INF


def exhaustive(c, R, param_bytes, repl, mem, limit, n_k, k0=0):
    N, K = c.shape
    order = sorted(range(N), key=lambda i: (-int(param_bytes[i]), i))         # largest first, then lower index
    plans = np.array(list(itertools.product(range(K), repeat=N)), dtype=np.int64)
    out, first = [], -1
    for t in range(n_k):
        marked = [i for i in order[: k0 + t] if param_bytes[i] > 0]
        cm = c.copy()
        for i in marked:
            cm[i, repl[i] != 0] = INF
        cost = np.zeros(len(plans), dtype=np.int64)
        for i in range(N):
            cost += cm[i, plans[:, i]]
        for i in range(N - 1):
            cost += R[i, plans[:, i], plans[:, i + 1]]
        cost = np.minimum(cost, INF)
        best = cost.min()
        cand = plans[cost == best]
        key = np.zeros(len(cand), dtype=np.int64)
        for i in range(N - 1, -1, -1):
            key = key * K + cand[:, i]
        plan = cand[np.argmin(key)]
        m = int(sum(mem[i, plan[i]] for i in range(N)))
        out.append((int(best), plan.astype(np.int32), m))
        if first < 0 and best < INF and m <= limit:
            first = t
    return out, first


@pytest.mark.parametrize("seed", range(8))
def test_against_exhaustive_search(seed):
    rng = np.random.default_rng(seed)
    N, K = int(rng.integers(2, 7)), int(rng.integers(2, 5))
    c = rng.integers(0, 50, size=(N, K)).astype(np.int64)
    R = rng.integers(0, 50, size=(N - 1, K, K)).astype(np.int64)
    param_bytes = rng.integers(0, 4, size=N).astype(np.int64) * 1000          # ties and operators without parameters
    repl = (rng.random((N, K)) < 0.5).astype(np.uint8)
    repl[:, 0] = 1                                                             # candidate 0 always replicates
    if seed % 2:
        repl[rng.integers(0, N)] = 1                                           # an operator that can only replicate
    mem = np.where(repl != 0, param_bytes[:, None], param_bytes[:, None] // 4).astype(np.int64)
    limit = int(mem.min(axis=1).sum() + rng.integers(0, 3000))
    n_k = N + 1
    want, want_first = exhaustive(c, R, param_bytes, repl, mem, limit, n_k)
    total, plan, plan_mem, first = oracle.memory_sweep(c, R, param_bytes, repl, mem, limit, n_k)
    for t in range(n_k):
        assert total[t] == want[t][0], t
        if total[t] < INF:                                   # without a feasible plan the walk means nothing
            assert plan_mem[t] == want[t][2] and np.array_equal(plan[t], want[t][1])
    assert first == want_first


def test_k0_and_plain_chain():
    rng = np.random.default_rng(11)
    N, K = 9, 6
    c = rng.integers(0, 100, size=(N, K)).astype(np.int64)
    R = rng.integers(0, 100, size=(N - 1, K, K)).astype(np.int64)
    pb = rng.integers(1, 1000, size=N).astype(np.int64)
    repl = (rng.random((N, K)) < 0.4).astype(np.uint8)
    mem = np.where(repl != 0, pb[:, None], pb[:, None] // 8).astype(np.int64)
    total, plan, plan_mem, first = oracle.memory_sweep(c, R, pb, repl, mem, 10**9, N + 1)
    arg, _, ctot, clast = oracle.chain(c[None], R[None])
    assert total[0] == ctot[0] and np.array_equal(plan[0], oracle.backtrack(arg, clast)[0]) and first == 0
    assert np.all(np.diff(total) >= 0)                       # removing candidates never makes the best plan cheaper
    t2, p2, m2, f2 = oracle.memory_sweep(c, R, pb, repl, mem, 10**9, 4, k0=3)
    assert np.array_equal(t2, total[3:7]) and np.array_equal(p2, plan[3:7]) and np.array_equal(m2, plan_mem[3:7])
    # with every parameter marked, no chosen candidate replicates a parameter
    assert all(repl[i, plan[N][i]] == 0 for i in range(N) if total[N] < INF)
    # an impossible limit: nothing is feasible
    assert oracle.memory_sweep(c, R, pb, repl, mem, -1, N + 1)[3] == -1
