"""Pins of the in-tree oracle (CPU only).

An in-tree generalises the cone of Sec. 4.3.2 (level 1): inner nodes may join several inputs too.  The oracle is
checked against exhaustive evaluation of the objective C of Sec. 4.2 with the tree's edges as E (all K^n plans),
against the chain oracle (a path is a tree), against the cone oracle (a root with chain branches), against closed
forms and against invariances that hold for any tree.
"""
import itertools

import numpy as np
import pytest

import oracle
from paper_2302_08141_amd.workloads import trees

INF = oracle.INF


def all_plans(parent, c, R):
    """Every assignment of every node: per root strategy the least objective, and overall the least objective with,
    among its plans, the smallest when compared from the last node backwards (consumers before their inputs)."""
    n, K = c.shape
    table = np.full(K, INF, dtype=np.int64)
    best = None
    for x in itertools.product(range(K), repeat=n):
        cost = sum(int(c[i, x[i]]) for i in range(n)) + sum(int(R[i, x[i], x[parent[i]]]) for i in range(n - 1))
        cost = min(cost, INF)
        table[x[n - 1]] = min(table[x[n - 1]], cost)
        key = (cost, tuple(reversed(x)))
        if best is None or key < best:
            best = key
    return table, best[0], np.array(tuple(reversed(best[1])), dtype=np.int32)


@pytest.mark.parametrize("seed", range(14))
def test_against_all_assignments(seed):
    rng = np.random.default_rng(seed)
    n = int(rng.integers(1, 8))
    K = int(rng.integers(2, 4)) if n > 5 else int(rng.integers(2, 5))
    parent = trees.random_tree(n, max_fan_in=3, chain_bias=0.4, seed=seed)
    hi = 3 if seed % 2 else 50                               # small range: ties everywhere
    c = rng.integers(0, hi, size=(n, K)).astype(np.int64)
    R = rng.integers(0, hi, size=(max(n - 1, 0), K, K)).astype(np.int64)
    if seed % 3 == 0:
        R[rng.random(R.shape) < 0.25] = INF
        c[rng.random(c.shape) < 0.1] = INF
    table, total, choice, plan, arg = oracle.tree(parent, c, R)
    want_table, want_total, want_plan = all_plans(parent, c, R)
    assert np.array_equal(table, want_table)
    assert total == want_total
    if total < INF:
        assert np.array_equal(plan, want_plan) and choice == want_plan[-1]
        # and the plan's objective, evaluated edge by edge, is the total
        assert sum(int(c[i, plan[i]]) for i in range(n)) + \
            sum(int(R[i, plan[i], plan[parent[i]]]) for i in range(n - 1)) == total
    else:
        assert choice == 0


def test_some_trees_join_inputs_below_the_root():
    # the generator really produces inner nodes with several inputs and depth >= 3 (what a root with chain
    # branches cannot express)
    found = 0
    for seed in range(14):
        parent = trees.random_tree(7, max_fan_in=3, chain_bias=0.4, seed=seed)
        fan = np.bincount(parent[:-1], minlength=7)
        found += int((fan[:-1] >= 2).any() and trees.depth(parent) >= 3)
    assert found >= 3


@pytest.mark.parametrize("seed", range(4))
def test_a_path_is_the_chain(seed):
    rng = np.random.default_rng(100 + seed)
    n, K = int(rng.integers(2, 12)), int(rng.integers(2, 9))
    parent = np.array(list(range(1, n)) + [-1], dtype=np.int32)
    c = rng.integers(0, 4, size=(n, K)).astype(np.int64)
    R = rng.integers(0, 4, size=(n - 1, K, K)).astype(np.int64)
    R[rng.random(R.shape) < 0.2] = INF
    table, total, choice, plan, arg = oracle.tree(parent, c, R)
    o_arg, o_vf, o_total, o_last = oracle.chain(c[None], R[None])
    assert total == o_total[0] and np.array_equal(table, o_vf[0])
    assert np.array_equal(arg, o_arg[0])
    if total < INF:
        assert choice == o_last[0] and np.array_equal(plan, oracle.backtrack(o_arg, o_last)[0])


@pytest.mark.parametrize("seed", range(4))
def test_a_root_with_chain_branches_is_the_cone(seed):
    rng = np.random.default_rng(200 + seed)
    K = int(rng.integers(2, 7))
    lens = [int(x) for x in rng.integers(1, 5, size=int(rng.integers(1, 5)))]
    n = sum(lens) + 1
    parent = np.full(n, -1, dtype=np.int32)
    c = rng.integers(0, 30, size=(n, K)).astype(np.int64)
    R = rng.integers(0, 30, size=(n - 1, K, K)).astype(np.int64)
    branches, at = [], 0
    for m in lens:                                           # branch = nodes at .. at+m-1, the last feeds the root
        parent[at:at + m] = np.arange(at + 1, at + m + 1)
        parent[at + m - 1] = n - 1
        branches.append((np.ascontiguousarray(c[at:at + m]), np.ascontiguousarray(R[at:at + m])))
        at += m
    table, total, choice, plan, _ = oracle.tree(parent, c, R)
    c_table, c_total, c_choice, c_plans = oracle.cone(branches, np.ascontiguousarray(c[n - 1]))
    assert np.array_equal(table, c_table) and total == c_total and choice == c_choice
    assert np.array_equal(plan[:-1], np.concatenate(c_plans))


def test_closed_forms_and_invariances():
    rng = np.random.default_rng(7)
    n, K = 9, 5
    parent = trees.random_tree(n, max_fan_in=3, chain_bias=0.3, seed=3)
    c = rng.integers(0, 1000, size=(n, K)).astype(np.int64)
    R = rng.integers(0, 1000, size=(n - 1, K, K)).astype(np.int64)
    # free edges: every node takes its own cheapest strategy
    _, total, _, plan, _ = oracle.tree(parent, c, np.zeros_like(R))
    assert total == c.min(axis=1).sum() and np.array_equal(plan, c.argmin(axis=1))
    # one candidate per node: the objective of the only plan
    _, total, _, _, _ = oracle.tree(parent, np.ascontiguousarray(c[:, :1]), np.ascontiguousarray(R[:, :1, :1]))
    assert total == c[:, 0].sum() + R[:, 0, 0].sum()
    # a node's costs shifted by a constant shift the total and every table entry, and move no choice
    table, total, choice, plan, _ = oracle.tree(parent, c, R)
    c2 = c.copy()
    c2[4] += 777
    table2, total2, choice2, plan2, _ = oracle.tree(parent, c2, R)
    assert total2 == total + 777 and np.array_equal(table2, table + 777) and np.array_equal(plan2, plan)
    # renumbering the nodes (any order that keeps inputs before consumers) changes nothing but the names
    order = [i for i in sorted(range(n - 1), key=lambda i: (trees.depth(parent) - _height(parent, i), -i))] + [n - 1]
    assert sorted(order) == list(range(n))
    new_of = np.empty(n, dtype=np.int64)
    new_of[order] = np.arange(n)
    parent3 = np.full(n, -1, dtype=np.int32)
    c3, R3 = np.empty_like(c), np.empty_like(R)
    for old in range(n):
        c3[new_of[old]] = c[old]
        if old < n - 1:
            parent3[new_of[old]] = new_of[parent[old]]
            R3[new_of[old]] = R[old]
    assert all(parent3[i] > i for i in range(n - 1))
    table3, total3, choice3, plan3, _ = oracle.tree(parent3, c3, R3)
    assert total3 == total and np.array_equal(table3, table) and np.array_equal(plan3[new_of], plan)
    # an infeasible root, a malformed parent array
    c4 = c.copy()
    c4[n - 1] = INF
    assert oracle.tree(parent, c4, R)[1] == INF
    with pytest.raises(ValueError):
        oracle.tree(np.array([1, 0, -1], dtype=np.int32), c[:3].copy(), R[:2].copy())


def _height(parent, i):
    """Edges from node i up to the root."""
    h = 0
    while parent[i] >= 0:
        i = parent[i]
        h += 1
    return h
