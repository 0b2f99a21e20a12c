"""Host arithmetic of rh_tree_plan (no GPU): runs, rounds and input lists of an in-tree."""
import ctypes

import numpy as np
import pytest

from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import trees


def plan(parent):
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    n = parent.shape[0]
    out = [np.full(n + 1, -7, dtype=np.int32) for _ in range(5)]
    n_runs = ctypes.c_int32(-1)
    hp = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    rounds = rh.lib().rh_tree_plan(n, hp(parent), *[hp(a) for a in out], ctypes.byref(n_runs))
    return rounds, n_runs.value, out


@pytest.mark.parametrize("seed", range(12))
def test_runs_and_rounds_of_random_trees(seed):
    n = [1, 2, 3, 9, 40, 200][seed % 6]
    parent = trees.random_tree(n, max_fan_in=1 + seed % 4, chain_bias=[0.0, 0.5, 0.9][seed % 3], seed=seed)
    rounds, n_runs, (first, last, round_start, child_start, child_list) = plan(parent)
    assert rounds >= 1 and 1 <= n_runs <= n
    # input lists: exactly the nodes whose parent is i, ascending
    for i in range(n):
        kids = child_list[child_start[i]:child_start[i + 1]].tolist()
        assert kids == [j for j in range(n) if parent[j] == i]
    # the runs partition the nodes into stretches of consecutive nodes...
    covered = []
    round_of_node = np.full(n, -1)
    assert round_start[0] == 0 and round_start[rounds] == n_runs
    for t in range(rounds):
        assert round_start[t] < round_start[t + 1]            # no empty round
        for u in range(round_start[t], round_start[t + 1]):
            f, e = int(first[u]), int(last[u])
            assert 0 <= f <= e < n
            covered += list(range(f, e + 1))
            round_of_node[f:e + 1] = t
            # ...inside which every node but the first has the node before it as its only input
            for i in range(f + 1, e + 1):
                assert [j for j in range(n) if parent[j] == i] == [i - 1]
            # and the first node does not continue the node before it
            kids_f = [j for j in range(n) if parent[j] == f]
            assert not (f > 0 and kids_f == [f - 1])
            # round = one more than the highest round among the runs that feed the first node
            want = 1 + max((round_of_node[j] for j in kids_f), default=-1)
            assert all(round_of_node[j] >= 0 for j in kids_f) and t == want
    assert sorted(covered) == list(range(n))
    assert round_of_node[n - 1] == rounds - 1                 # the root comes last


def test_a_path_is_one_run_and_a_star_two_rounds():
    rounds, n_runs, (first, last, *_rest) = plan(list(range(1, 50)) + [-1])
    assert (rounds, n_runs, first[0], last[0]) == (1, 1, 0, 49)
    rounds, n_runs, (first, last, round_start, *_r) = plan([5, 5, 5, 5, 5, -1])
    assert (rounds, n_runs) == (2, 6) and round_start[:3].tolist() == [0, 5, 6]
    assert (first[5], last[5]) == (5, 5)
    # a root whose only input is not the node before it starts a run of its own
    rounds, n_runs, _ = plan([2, 2, 3, -1])
    assert (rounds, n_runs) == (2, 3)                          # runs {0}, {1}, then {2, 3}


def test_malformed_parent_arrays_are_refused():
    assert plan([1, 0, -1])[0] == -2                           # an input after its consumer
    assert plan([1, 2, 2])[0] == -2                            # the last node is not the root
    assert plan([-1, 2, -1])[0] == -2                          # a second root
    assert plan([3, 2, -1])[0] == -2                           # out of range
    L = rh.lib()
    assert L.rh_tree_plan(0, None, None, None, None, None, None, None) == -2
    assert L.rh_tree_plan(3, None, None, None, None, None, None, None) == -1
    # argument errors of rh_tree_dp are found before anything touches a device
    rs = np.array([0, 1], dtype=np.int32)
    hp = rs.ctypes.data_as(ctypes.c_void_p)
    assert L.rh_tree_dp(1, 4, 48, 1, 1, hp, None, None, None, None, None, None, 0, None, 0, None, None, None, None,
                        None, None) == -3
    assert L.rh_tree_dp(1, 4, 64, 1, 1, hp, None, None, None, None, None, None, 0, None, 0, None, None, None, None,
                        None, None) == -1
    assert L.rh_tree_dp(1, 4, 64, 5, 1, hp, None, None, None, None, None, None, 0, None, 0, None, None, None, None,
                        None, None) == -2                      # more runs than nodes
    assert L.rh_tree_dp(1, 4, 64, 2, 1, hp, None, None, None, None, None, None, 0, None, 0, None, None, None, None,
                        None, None) == -2                      # the rounds do not cover the runs
    assert L.rh_tree_dp(0, 4, 64, 1, 1, hp, None, None, None, None, None, None, 0, None, 0, None, None, None, None,
                        None, None) == 0
