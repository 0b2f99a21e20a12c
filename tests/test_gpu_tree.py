"""GPU parity of the in-tree dynamic program (rh_tree_plan + rh_tree_dp) against the CPU oracle (bit-exact)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import synthetic as syn, trees

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
INF = oracle.INF


def gpu_tree(parent, c, R, shared_R=False):
    """c[B][n][Kp]; R[B][n-1][Kp][Kp] or [n-1][Kp][Kp] with shared_R."""
    B, n, Kp = c.shape
    tp = rh.TreePlan(parent, DEV)
    arg = torch.full((B, max(n - 1, 0), Kp), -1, dtype=torch.int16, device=DEV)
    w = torch.full((B, n, Kp), -5, dtype=torch.int64, device=DEV)
    total = torch.full((B,), -5, dtype=torch.int64, device=DEV)
    choice = torch.full((B,), -5, dtype=torch.int32, device=DEV)
    plan = torch.full((B, n), -5, dtype=torch.int32, device=DEV)
    dR = torch.from_numpy(R).to(DEV) if n > 1 else None
    rh.rh_tree_dp(B, Kp, tp, torch.from_numpy(c).to(DEV), n * Kp, dR, 0 if shared_R else (n - 1) * Kp * Kp,
                  arg if n > 1 else None, w, total, choice, plan)
    torch.cuda.synchronize()
    return tp, arg.cpu().numpy().view(np.uint16), w.cpu().numpy(), total.cpu().numpy(), choice.cpu().numpy(), \
        plan.cpu().numpy()


def check(parent, c, R, shared_R=False):
    tp, arg, w, total, choice, plan = gpu_tree(parent, c, R, shared_R)
    for p in range(c.shape[0]):
        o_table, o_total, o_choice, o_plan, o_arg = oracle.tree(parent, np.ascontiguousarray(c[p]),
                                                                R if shared_R else np.ascontiguousarray(R[p]))
        assert total[p] == o_total and choice[p] == o_choice, p
        assert np.array_equal(w[p, -1], o_table)
        assert np.array_equal(arg[p], o_arg)
        assert np.array_equal(plan[p], o_plan)
    return tp, total


@pytest.mark.parametrize("Kp,n,fan,seed", [(16, 30, 4, 0), (32, 61, 3, 1), (64, 200, 4, 2), (64, 333, 2, 3),
                                           (128, 90, 4, 4), (256, 70, 3, 5), (512, 12, 2, 6), (1024, 8, 3, 9)])
def test_random_trees(Kp, n, fan, seed):
    parent = trees.random_tree(n, max_fan_in=fan, chain_bias=0.55, seed=seed)
    counts = np.bincount(parent[:-1], minlength=n)
    assert trees.depth(parent) >= 3 and counts.max() >= 2 and (counts[:-1] >= 2).any()   # joins below the root
    K = Kp if seed % 2 else Kp - Kp // 5
    B = 3 if Kp <= 256 else 1
    cs, Rs = [], []
    for p in range(B):
        c, R = trees.random_tree_costs(parent, K, Kp, seed=seed * 10 + p, infeasible=0.15 if p == 1 else 0.0,
                                       ragged=(p == 2))
        if p == 2:                                            # ties everywhere
            c = np.where(c < INF, c % 3, INF)
            R = np.where(R < INF, R % 3, INF)
        cs.append(c)
        Rs.append(R)
    tp, total = check(parent, np.stack(cs), np.stack(Rs))
    assert tp.n_rounds >= 2 and (total < INF).any()


def test_one_table_set_for_all_problems_and_a_dead_tree():
    parent = trees.random_tree(120, max_fan_in=4, chain_bias=0.5, seed=11)
    Kp = 64
    c0, R = trees.random_tree_costs(parent, 50, Kp, seed=5)
    cs = np.stack([c0, np.where(c0 < INF, c0 // 2, INF), c0.copy()])
    cs[2, 77, :] = INF                                        # an operator without a feasible strategy
    tp, total = check(parent, cs, R, shared_R=True)
    assert total[2] == INF and total[0] < INF


def test_a_path_is_the_chain_call():
    n, Kp = 400, 128
    c, R = syn.random_chain_batch([3, 4], n, 100, 1_000_000, 10_000_000, Kp=Kp)
    parent = np.array(list(range(1, n)) + [-1], dtype=np.int32)
    tp, arg, w, total, choice, plan = gpu_tree(parent, c, R)
    assert (tp.n_rounds, tp.n_runs) == (1, 1)
    dc, dR = torch.from_numpy(c).to(DEV), torch.from_numpy(R).to(DEV)
    c_arg = torch.empty((2, n - 1, Kp), dtype=torch.int16, device=DEV)
    c_vf = torch.empty((2, Kp), dtype=torch.int64, device=DEV)
    c_total = torch.empty(2, dtype=torch.int64, device=DEV)
    c_last = torch.empty(2, dtype=torch.int32, device=DEV)
    c_plan = torch.empty((2, n), dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain(2, n, Kp, dc, n * Kp, dR, (n - 1) * Kp * Kp, c_arg, c_vf, c_total, c_last)
    rh.rh_backtrack(2, n, Kp, c_arg, c_last, c_plan)
    torch.cuda.synchronize()
    assert np.array_equal(total, c_total.cpu().numpy()) and np.array_equal(choice, c_last.cpu().numpy())
    assert np.array_equal(arg, c_arg.cpu().numpy().view(np.uint16)) and np.array_equal(w[:, -1], c_vf.cpu().numpy())
    assert np.array_equal(plan, c_plan.cpu().numpy())
    o_arg, _, o_total, _ = oracle.chain(c, R)
    assert np.array_equal(total, o_total) and np.array_equal(arg, o_arg)


def test_single_node_long_runs_and_no_plan():
    rng = np.random.default_rng(3)
    c = rng.integers(0, 100, size=(2, 1, 64)).astype(np.int64)
    c[1, 0, :5] = INF
    check(np.array([-1], dtype=np.int32), c, np.zeros((2, 0, 64, 64), dtype=np.int64))
    # a comb: a long run that every second node of another long run joins
    n = 600
    parent = trees.random_tree(n, max_fan_in=2, chain_bias=0.93, seed=9)
    c, R = trees.random_tree_costs(parent, 64, 64, seed=2, infeasible=0.05)
    tp, _ = check(parent, c[None], R[None])
    assert (tp.host["run_last"][:tp.n_runs] - tp.host["run_first"][:tp.n_runs]).max() >= 20
    # plan = None: totals only
    tp = rh.TreePlan(parent, DEV)
    w = torch.empty((1, n, 64), dtype=torch.int64, device=DEV)
    arg = torch.empty((1, n - 1, 64), dtype=torch.int16, device=DEV)
    total = torch.empty(1, dtype=torch.int64, device=DEV)
    choice = torch.empty(1, dtype=torch.int32, device=DEV)
    rh.rh_tree_dp(1, 64, tp, torch.from_numpy(c[None]).to(DEV), n * 64, torch.from_numpy(R[None]).to(DEV),
                  (n - 1) * 64 * 64, arg, w, total, choice, None)
    torch.cuda.synchronize()
    assert total.item() == oracle.tree(parent, c, R)[1]


def test_the_bench_tree_at_full_size():
    # 4096 nodes, 64 strategies, inner nodes joining up to four inputs: the tree the timing row uses, two problems
    # sharing its tables (the second with halved node costs), every output against the oracle
    n, K = 4096, 64
    parent = trees.random_tree(n, max_fan_in=4, chain_bias=0.7)
    c, R = trees.random_tree_costs(parent, K)
    tp, total = check(parent, np.stack([c, c // 2]), R, shared_R=True)
    assert tp.n_rounds >= 20 and trees.depth(parent) >= 40 and (total < INF).all()
