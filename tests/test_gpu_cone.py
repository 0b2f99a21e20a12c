"""GPU parity of the cone DP (branch batch through the chain DP, then rh_cone_merge) against the CPU oracle."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import cones as wc

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
INF = oracle.INF


def gpu_cones(pk):
    c, R = torch.from_numpy(pk["c"]).to(DEV), torch.from_numpy(pk["R"]).to(DEV)
    Bb, N, Kp = pk["c"].shape
    n_cones = len(pk["c_root"])
    arg = torch.empty((Bb, N - 1, Kp), dtype=torch.int16, device=DEV)
    w = torch.empty((Bb, Kp), dtype=torch.int64, device=DEV)
    tot_b = torch.empty(Bb, dtype=torch.int64, device=DEV)
    last_b = torch.empty(Bb, dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain(Bb, N, Kp, c, N * Kp, R, (N - 1) * Kp * Kp, arg, w, tot_b, last_b)
    table = torch.full((n_cones, Kp), -7, dtype=torch.int64, device=DEV)
    total = torch.full((n_cones,), -7, dtype=torch.int64, device=DEV)
    choice = torch.full((n_cones,), -7, dtype=torch.int32, device=DEV)
    branch_last = torch.full((Bb,), -7, dtype=torch.int32, device=DEV)
    rh.rh_cone_merge(n_cones, Bb, Kp, torch.from_numpy(pk["branch_start"]).to(DEV), w,
                     torch.from_numpy(pk["c_root"]).to(DEV), table, total, choice, branch_last)
    plan = torch.empty((Bb, N), dtype=torch.int32, device=DEV)
    rh.rh_backtrack(Bb, N, Kp, arg, branch_last, plan)
    torch.cuda.synchronize()
    return table.cpu().numpy(), total.cpu().numpy(), choice.cpu().numpy(), plan.cpu().numpy()


@pytest.mark.parametrize("K,Kp,n_cones,infeasible", [(4, 16, 50, 0.0), (13, 16, 40, 0.2), (64, 64, 300, 0.0),
                                                      (100, 128, 30, 0.1), (256, 256, 6, 0.0)])
def test_random_cones(K, Kp, n_cones, infeasible):
    cones = wc.random_cones(n_cones, K, max_branches=5, max_len=6, seed=K * 7 + n_cones, infeasible=infeasible)
    if K == 13:
        cones[3][1][:] = INF                               # a root without a feasible strategy
        cones[5] = (cones[5][0], np.zeros(K, dtype=np.int64))
    pk = wc.pack(cones, Kp)
    table, total, choice, plan = gpu_cones(pk)
    N = pk["N"]
    b = 0
    for q, (branches, c_root) in enumerate(cones):
        cr = np.full(Kp, INF, dtype=np.int64)
        cr[:K] = c_root
        pb = [(np.ascontiguousarray(np.pad(cb, ((0, 0), (0, Kp - K)), constant_values=INF)),
               np.ascontiguousarray(np.pad(Rb, ((0, 0), (0, Kp - K), (0, Kp - K)), constant_values=INF)))
              for cb, Rb in branches]
        o_table, o_total, o_choice, o_plans = oracle.cone(pb, cr)
        assert np.array_equal(table[q], o_table), q
        assert total[q] == o_total and choice[q] == o_choice
        for (cb, _), op in zip(branches, o_plans):
            n = cb.shape[0]
            assert plan[b, N - 1] == o_choice
            assert np.array_equal(plan[b, N - 1 - n:N - 1], op), (q, b)
            b += 1


def test_cone_without_branches_and_argument_errors():
    Kp = 64
    c_root = torch.arange(Kp, 0, -1, dtype=torch.int64, device=DEV).reshape(1, Kp).contiguous()
    start = torch.zeros(2, dtype=torch.int32, device=DEV)
    total = torch.zeros(1, dtype=torch.int64, device=DEV)
    choice = torch.zeros(1, dtype=torch.int32, device=DEV)
    rh.rh_cone_merge(1, 0, Kp, start, None, c_root, None, total, choice, None)
    torch.cuda.synchronize()
    assert total.item() == 1 and choice.item() == Kp - 1
    L = rh.lib()
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    assert L.rh_cone_merge(1, 0, 48, P(start), None, P(c_root), None, P(total), P(choice), None, None) == -3
    assert L.rh_cone_merge(-1, 0, 64, P(start), None, P(c_root), None, P(total), P(choice), None, None) == -2
    assert L.rh_cone_merge(1, 2, 64, P(start), None, P(c_root), None, P(total), P(choice), None, None) == -1
    assert L.rh_cone_merge(0, 0, 64, None, None, None, None, None, None, None, None) == 0


def test_the_table_of_a_cone_is_the_first_row_of_the_chain_above_it():
    # every root strategy is kept for the next level (Sec. 4.3.2): a cone whose root feeds a chain of further
    # operators.  The cone's table takes the place of the node costs of the chain's first operator, the chain's
    # backtrack gives the root's strategy, and that starts the branches' backtrack.  Checked against the in-tree
    # oracle on the whole graph.
    K = Kp = 64
    rng = np.random.default_rng(21)
    (branches, c_root), = wc.random_cones(1, K, max_branches=4, max_len=5, seed=99)
    pk = wc.pack([(branches, c_root)], Kp)
    c, R = torch.from_numpy(pk["c"]).to(DEV), torch.from_numpy(pk["R"]).to(DEV)
    Bb, N, _ = pk["c"].shape
    arg = torch.empty((Bb, N - 1, Kp), dtype=torch.int16, device=DEV)
    w = torch.empty((Bb, Kp), dtype=torch.int64, device=DEV)
    tot_b = torch.empty(Bb, dtype=torch.int64, device=DEV)
    last_b = torch.empty(Bb, dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain(Bb, N, Kp, c, N * Kp, R, (N - 1) * Kp * Kp, arg, w, tot_b, last_b)
    table = torch.empty((1, Kp), dtype=torch.int64, device=DEV)
    total = torch.empty(1, dtype=torch.int64, device=DEV)
    choice = torch.empty(1, dtype=torch.int32, device=DEV)
    rh.rh_cone_merge(1, Bb, Kp, torch.from_numpy(pk["branch_start"]).to(DEV), w, torch.from_numpy(pk["c_root"]).to(DEV),
                     table, total, choice, None)
    # the chain above the root: M further operators; operator 0 of that chain is the root with the table as costs
    M = 6
    up_c = rng.integers(0, 2000, size=(M, K)).astype(np.int64)
    up_R = rng.integers(0, 10000, size=(M, K, K)).astype(np.int64)
    cc = torch.cat([table, torch.from_numpy(up_c).to(DEV)]).reshape(1, M + 1, Kp).contiguous()
    c_arg = torch.empty((1, M, Kp), dtype=torch.int16, device=DEV)
    c_total = torch.empty(1, dtype=torch.int64, device=DEV)
    c_last = torch.empty(1, dtype=torch.int32, device=DEV)
    c_plan = torch.empty((1, M + 1), dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain(1, M + 1, Kp, cc, (M + 1) * Kp, torch.from_numpy(up_R[None]).to(DEV), M * Kp * Kp, c_arg, None,
                        c_total, c_last)
    rh.rh_backtrack(1, M + 1, Kp, c_arg, c_last, c_plan)
    branch_last = c_plan[:, 0].expand(Bb).contiguous()       # the root's strategy, for every branch
    plan = torch.empty((Bb, N), dtype=torch.int32, device=DEV)
    rh.rh_backtrack(Bb, N, Kp, arg, branch_last, plan)
    torch.cuda.synchronize()
    # the same graph as one in-tree: the branches' nodes, the root, then the chain above it
    lens = [cb.shape[0] for cb, _ in branches]
    n = sum(lens) + 1 + M
    root = sum(lens)
    parent = np.full(n, -1, dtype=np.int32)
    tc = np.zeros((n, K), dtype=np.int64)
    tR = np.zeros((n - 1, K, K), dtype=np.int64)
    at = 0
    for cb, Rb in branches:
        m = cb.shape[0]
        parent[at:at + m] = np.arange(at + 1, at + m + 1)
        parent[at + m - 1] = root
        tc[at:at + m], tR[at:at + m] = cb, Rb
        at += m
    tc[root] = c_root
    parent[root:n - 1] = np.arange(root + 1, n)
    tc[root + 1:] = up_c
    tR[root:] = up_R
    o_table, o_total, o_choice, o_plan, _ = oracle.tree(parent, tc, tR)
    assert c_total.item() == o_total and c_last.item() == o_choice
    got = c_plan.cpu().numpy()[0]
    assert np.array_equal(got, o_plan[root:])
    at = 0
    for b, m in enumerate(lens):
        assert np.array_equal(plan[b, N - 1 - m:N - 1].cpu().numpy(), o_plan[at:at + m]), b
        at += m
