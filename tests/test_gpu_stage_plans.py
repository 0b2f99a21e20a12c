"""GPU parity of rh_stage_plans (the plans of all chosen stages at once) against the CPU oracle: every stage is
the chain oracle on its slice of the chain, its total the entry of the oracle's table of stage times."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import synthetic as syn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
INF = oracle.INF


def gpu_plans(bounds, c, R, want_plan=True):
    B, L, Kp = c.shape
    S = bounds.shape[1] - 1
    arg = torch.full((B, max(L - 1, 0), Kp), -1, dtype=torch.int16, device=DEV)
    total = torch.full((B, S), -7, dtype=torch.int64, device=DEV)
    last = torch.full((B, S), -7, dtype=torch.int32, device=DEV)
    plan = torch.full((B, L), -7, dtype=torch.int32, device=DEV) if want_plan else None
    rh.rh_stage_plans(B, L, Kp, S, torch.from_numpy(bounds).to(DEV), torch.from_numpy(c).to(DEV),
                      torch.from_numpy(R).to(DEV) if L > 1 else None, arg if L > 1 else None, total, last, plan)
    torch.cuda.synchronize()
    return (arg.cpu().numpy().view(np.uint16), total.cpu().numpy(), last.cpu().numpy(),
            plan.cpu().numpy() if want_plan else None)


def check(bounds, c, R):
    B, L, Kp = c.shape
    S = bounds.shape[1] - 1
    arg, total, last, plan = gpu_plans(bounds, c, R)
    covered = np.zeros((B, L), bool)
    for p in range(B):
        for t in range(S):
            f, e1 = int(bounds[p, t]), int(bounds[p, t + 1])
            if not (0 <= f < e1 <= L):
                assert total[p, t] == INF and last[p, t] == 0
                continue
            o_arg, _, o_total, o_last = oracle.chain(np.ascontiguousarray(c[p:p + 1, f:e1]),
                                                     np.ascontiguousarray(R[p:p + 1, f:e1 - 1]))
            assert total[p, t] == o_total[0] and last[p, t] == o_last[0], (p, t)
            assert np.array_equal(arg[p, f:e1 - 1], o_arg[0]), (p, t)
            assert np.array_equal(plan[p, f:e1], oracle.backtrack(o_arg, o_last)[0]), (p, t)
            covered[p, f:e1] = True
    assert (plan[~covered] == -1).all()
    return total


@pytest.mark.parametrize("Kp,L,S,B", [(16, 40, 5, 2), (32, 1, 1, 1), (64, 300, 17, 3), (64, 64, 64, 1), (128, 150, 4, 2),
                                      (256, 90, 7, 1), (512, 10, 3, 1), (1024, 6, 2, 1)])
def test_ragged_stages(Kp, L, S, B):
    rng = np.random.default_rng(Kp + L)
    K = Kp - Kp // 5 if L % 2 else Kp
    c, R = syn.random_chain_batch(range(B), L, K, 1000, 5000, Kp=Kp)
    if B > 1:                                                 # ties everywhere in the second problem
        c[1] = np.where(c[1] < INF, c[1] % 3, INF)
        R[1] = np.where(R[1] < INF, R[1] % 3, INF)
    if B > 2:                                                 # infeasible pairs, and an operator that cannot run
        R[2][rng.random(R[2].shape) < 0.2] = INF
        c[2, L // 2, :] = INF
    bounds = np.zeros((B, S + 1), np.int32)
    for p in range(B):
        cuts = np.sort(rng.choice(np.arange(1, L), size=S - 1, replace=False)) if S > 1 else np.zeros(0, np.int32)
        bounds[p] = np.concatenate([[0], cuts, [L]])
    total = check(bounds, c, R)
    if B > 2:
        assert (total[2] == INF).any()


def test_stages_found_by_the_search_and_their_table_entries():
    # table of stage times -> search -> the plans of the stages it chose: every stage's total is its table entry,
    # the largest one the bottleneck
    L, K, S = 700, 64, 9
    c, R = syn.random_chain_batch([21], L, K, 100_000, 200_000)
    ldT = L + 2
    d_c, d_R = torch.from_numpy(c).to(DEV), torch.from_numpy(R).to(DEV)
    T = torch.empty((1, L, ldT), dtype=torch.int64, device=DEV)
    rh.rh_interval_costs(1, L, K, d_c, d_R, ldT, T)
    bott = torch.empty((1, S), dtype=torch.int64, device=DEV)
    cut = torch.empty((1, S, L + 1), dtype=torch.int32, device=DEV)
    bounds = torch.empty((1, S + 1), dtype=torch.int32, device=DEV)
    ws = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP_INTERVAL, 1, L, S), dtype=torch.uint8, device=DEV)
    rh.rh_stage_dp_interval(1, L, S, ldT, T, bott, cut, S, bounds, ws)
    torch.cuda.synchronize()
    o_T = oracle.interval_costs(c[0], R[0], ldT=ldT, nthreads=8)
    o_b, _, o_bounds = oracle.stage_interval(o_T[None], S, s_query=S, nthreads=4)
    assert np.array_equal(bounds.cpu().numpy(), o_bounds)
    total = check(o_bounds, c, R)
    assert [int(x) for x in total[0]] == [int(o_T[o_bounds[0, t], o_bounds[0, t + 1]]) for t in range(S)]
    assert total[0].max() == o_b[0, S - 1]


def test_stage_partition_size():
    # 4096 operators with 64 strategies in 64 stages of very different length (one of a single operator, one of 900)
    L, K, S = 4096, 64, 64
    c, R = syn.random_chain_batch([11], L, K, 100_000, 200_000)
    rng = np.random.default_rng(8)
    cuts = np.sort(rng.choice(np.arange(902, L), size=S - 3, replace=False))
    bounds = np.concatenate([[0, 1, 901], cuts, [L]]).astype(np.int32)[None]
    check(bounds, c, R)


def test_boundaries_that_describe_no_stage_and_totals_only():
    L, Kp = 50, 64
    c, R = syn.random_chain_batch([4, 5], L, 60, 1000, 5000, Kp=Kp)
    bounds = np.array([[-1, -1, -1, -1], [0, 20, 20, 50]], np.int32)       # no split found; an empty stage
    check(bounds, c, R)
    arg, total, last, plan = gpu_plans(np.array([[0, 10, 50], [0, 49, 50]], np.int32), c, R, want_plan=False)
    for p, (a, b) in enumerate([(0, 10), (0, 49)]):
        assert total[p, 0] == oracle.chain(np.ascontiguousarray(c[p:p + 1, a:b]), np.ascontiguousarray(R[p:p + 1, a:b - 1]))[2][0]


def test_argument_errors():
    lib = rh.lib()
    t = torch.zeros(1 << 14, dtype=torch.int64, device=DEV)
    P = ctypes.c_void_p(t.data_ptr())
    call = lambda **kw: lib.rh_stage_plans(kw.get("B", 1), kw.get("L", 8), kw.get("Kp", 16), kw.get("S", 2),
                                           kw.get("bounds", P), kw.get("c", P), kw.get("R", P), kw.get("arg", P), P, P,
                                           None, None)
    assert call(S=9) == -2 and call(S=0) == -2 and call(L=0) == -2 and call(B=-1) == -2 and call(Kp=48) == -3
    assert call(bounds=None) == -1 and call(c=None) == -1 and call(R=None) == -1 and call(arg=None) == -1
    assert call(c=ctypes.c_void_p(t.data_ptr() + 8)) == -2
    assert call(B=0, bounds=None, c=None) == 0
    torch.cuda.synchronize()
