"""Pins of the cone oracle (CPU only).

A cone is one root with several inputs whose other nodes have one input each
(Sec. 4.3.2, level 1).  The oracle is checked against exhaustive evaluation of
the objective C of Sec. 4.2 on the cone's tree edges, against the chain oracle
on a one-branch cone, and against closed forms.
"""
import itertools

import numpy as np
import pytest

import oracle

INF = oracle.INF


def all_plans(branches, c_root):
    """min over every assignment of every node, per root strategy; and the best assignment overall
    (root lowest, then each branch smallest when compared from its last operator backwards)."""
    K = len(c_root)
    table = np.full(K, INF, dtype=np.int64)
    best_plans = {}
    for r in range(K):
        tot = min(int(c_root[r]), INF)
        plans = []
        for cb, Rb in branches:
            n = cb.shape[0]
            best, bestp = None, None
            for x in itertools.product(range(K), repeat=n):
                cost = sum(int(cb[i, x[i]]) for i in range(n))
                cost += sum(int(Rb[i, x[i], x[i + 1]]) for i in range(n - 1)) + int(Rb[n - 1, x[n - 1], r])
                cost = min(cost, INF)
                key = (cost, tuple(reversed(x)))
                if best is None or key < best:
                    best, bestp = key, x
            tot = min(tot + best[0], INF)
            plans.append(np.array(bestp, dtype=np.int32))
        table[r] = tot
        best_plans[r] = plans
    r_star = int(np.argmin(table))
    return table, int(table[r_star]), r_star, best_plans[r_star]


@pytest.mark.parametrize("seed", range(10))
def test_against_all_assignments(seed):
    rng = np.random.default_rng(seed)
    K = int(rng.integers(2, 5))
    n_br = int(rng.integers(1, 4))
    hi = 3 if seed % 2 else 40                       # small range: many ties
    branches = []
    for _ in range(n_br):
        n = int(rng.integers(1, 5))
        cb = rng.integers(0, hi, size=(n, K)).astype(np.int64)
        Rb = rng.integers(0, hi, size=(n, K, K)).astype(np.int64)
        if seed % 3 == 0:
            Rb[rng.random(Rb.shape) < 0.25] = INF
        branches.append((cb, Rb))
    c_root = rng.integers(0, hi, size=K).astype(np.int64)
    if seed == 6:
        c_root[0] = INF
    want = all_plans(branches, c_root)
    table, total, choice, plans = oracle.cone(branches, c_root)
    assert np.array_equal(table, want[0]) and total == want[1] and choice == want[2]
    for got, exp in zip(plans, want[3]):
        assert np.array_equal(got, exp)


def test_one_branch_is_a_chain_and_no_branch_is_the_root_alone():
    rng = np.random.default_rng(3)
    K, n = 6, 5
    cb = rng.integers(0, 100, size=(n, K)).astype(np.int64)
    Rb = rng.integers(0, 100, size=(n, K, K)).astype(np.int64)
    c_root = rng.integers(0, 100, size=K).astype(np.int64)
    table, total, choice, plans = oracle.cone([(cb, Rb)], c_root)
    c = np.concatenate([cb, c_root[None]])[None]
    arg, vfinal, ctot, clast = oracle.chain(np.ascontiguousarray(c), np.ascontiguousarray(Rb[None]))
    assert np.array_equal(table, vfinal[0]) and total == ctot[0] and choice == clast[0]
    assert np.array_equal(plans[0], oracle.backtrack(arg, clast)[0, :-1])
    t0, tot0, ch0, p0 = oracle.cone([], c_root)
    assert np.array_equal(t0, c_root) and tot0 == c_root.min() and ch0 == int(c_root.argmin()) and p0 == []


def test_branches_add_up():
    # identical branches: the table is the root cost plus m times one branch's contribution
    rng = np.random.default_rng(4)
    K = 5
    cb = rng.integers(0, 50, size=(3, K)).astype(np.int64)
    Rb = rng.integers(0, 50, size=(3, K, K)).astype(np.int64)
    zero = np.zeros(K, dtype=np.int64)
    one, *_ = oracle.cone([(cb, Rb)], zero)
    for m in (2, 5):
        c_root = rng.integers(0, 50, size=K).astype(np.int64)
        table, *_ = oracle.cone([(cb, Rb)] * m, c_root)
        assert np.array_equal(table, c_root + m * one)
