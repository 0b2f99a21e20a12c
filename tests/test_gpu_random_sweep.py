"""Seeded random shapes through every route of the chain DP, the tree DP, the stage searches and the table of
stage times, each compared with the CPU oracle bit for bit: shapes no hand-picked case names (ragged candidate
counts, ties, infeasible entries, tile edges, every workspace kind that the sizes allow)."""
import numpy as np
import pytest
import torch

import oracle
import test_gpu_fused
import test_gpu_stage
import test_gpu_stage_plans
import test_gpu_stage_window
import test_gpu_tree
from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import specs as sp, trees

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
INF = oracle.INF


def rand_chain(rng, B, N, K, Kp, small, inf_p):
    hi_c, hi_r = (3, 3) if small else (1000, 5000)
    c = np.full((B, N, Kp), INF, np.int64)
    R = np.full((B, max(N - 1, 0), Kp, Kp), INF, np.int64)
    c[:, :, :K] = rng.integers(0, hi_c, size=(B, N, K))
    R[:, :, :K, :K] = rng.integers(0, hi_r, size=(B, max(N - 1, 0), K, K))
    if inf_p > 0:
        R[rng.random(R.shape) < inf_p] = INF
        dead = rng.random(c.shape) < inf_p / 2
        dead[:, :, 0] = False
        c[dead] = INF
    return c, R


def chain_case(rng):
    Kp = int(rng.choice([16, 32, 64, 128, 256, 512, 1024]))
    big = Kp >= 512
    B = int(rng.integers(1, 4 if big else 40))
    N = int(rng.integers(1, 12 if big else (400 if Kp <= 64 else 160)))
    if B * N * Kp * Kp > 6e7:
        N = max(1, int(6e7 / (B * Kp * Kp)))
    K = int(rng.integers(max(1, Kp // 2), Kp + 1))
    c, R = rand_chain(rng, B, N, K, Kp, rng.random() < 0.4, float(rng.choice([0, 0, 0.1, 0.4])))
    which = (None, rh.WS_MINPLUS_CHAIN, rh.WS_MINPLUS_CHAIN_SEGMENTED)[int(rng.integers(0, 3))]
    need = rh.rh_workspace_size(which, B, N, Kp) if which is not None else 0
    ws = torch.empty(need, dtype=torch.uint8, device=DEV) if need else None
    dc = torch.from_numpy(c).to(DEV)
    dR = torch.from_numpy(R).to(DEV) if N > 1 else None
    arg = torch.full((B, max(N - 1, 0), Kp), -1, dtype=torch.int16, device=DEV)
    vf = torch.zeros((B, Kp), dtype=torch.int64, device=DEV)
    total = torch.zeros(B, dtype=torch.int64, device=DEV)
    last = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    plan = torch.full((B, N), -1, dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain(B, N, Kp, dc, N * Kp, dR, (N - 1) * Kp * Kp, arg if N > 1 else None, vf, total, last, ws)
    rh.rh_backtrack(B, N, Kp, arg if N > 1 else None, last, plan)
    torch.cuda.synchronize()
    o_arg, o_vf, o_total, o_last = oracle.chain(c, R, nthreads=8)
    assert np.array_equal(total.cpu().numpy(), o_total) and np.array_equal(last.cpu().numpy(), o_last)
    assert np.array_equal(vf.cpu().numpy(), o_vf)
    assert np.array_equal(arg.cpu().numpy().view(np.uint16), o_arg)
    assert np.array_equal(plan.cpu().numpy(), oracle.backtrack(o_arg, o_last))


def tree_case(rng):
    Kp = int(rng.choice([16, 32, 64, 128, 256, 512, 1024]))
    n = int(rng.integers(1, 400 if Kp <= 64 else (120 if Kp <= 256 else 12)))
    B = int(rng.integers(1, 4))
    K = int(rng.integers(max(1, Kp // 2), Kp + 1))
    seed = int(rng.integers(0, 1 << 30))
    parent = trees.random_tree(n, max_fan_in=int(rng.integers(2, 6)), chain_bias=float(rng.choice([0.2, 0.55, 0.8])),
                               seed=seed)
    cs, Rs = [], []
    for p in range(B):
        c, R = trees.random_tree_costs(parent, K, Kp, seed=seed + p, infeasible=float(rng.choice([0, 0.15])),
                                       ragged=bool(rng.integers(0, 2)))
        if rng.random() < 0.4:                                # ties everywhere
            c, R = np.where(c < INF, c % 3, INF), np.where(R < INF, R % 3, INF)
        cs.append(c)
        Rs.append(R)
    test_gpu_tree.check(parent, np.stack(cs), np.stack(Rs))


def window_case(rng):
    L = int(rng.integers(1, 3000))
    S = int(rng.integers(1, min(L, 64) + 1))
    B = int(rng.integers(1, 4))
    mode = int(rng.integers(0, 3))
    cost = rng.integers(0, 3 if mode == 0 else 100000, size=(B, L)).astype(np.int64)
    if mode == 2:                                             # a few segments a thousand times heavier
        cost[:, rng.choice(L, size=max(1, L // 50), replace=False)] *= 1000
    xfer = rng.integers(0, 20000, size=(B, L + 1)).astype(np.int64) if rng.random() < 0.7 else None
    num, den = [(-1, 1), (0, 1), (1, 8), (1, 2), (1, 1), (5, 2), (20, 1)][int(rng.integers(0, 7))]
    test_gpu_stage_window.check(cost, S, xfer, num, den)


def stage_case(rng):
    L = int(rng.integers(1, 9000))
    S = int(rng.integers(1, min(L, 40) + 1))
    cost = rng.integers(0, 3 if rng.random() < 0.3 else 100000, size=(int(rng.integers(1, 3)), L)).astype(np.int64)
    test_gpu_stage.check(cost, S, int(rng.integers(0, S + 1)))


def search_case(rng):
    L = int(rng.integers(1, 1500))
    B = int(rng.choice([1, 2, 3, 40]))                       # 40 problems: the rows of a column stay in one workgroup
    if B == 40:
        L = min(L, 300)
    S = int(rng.integers(1, min(L, 64) + 1))
    ldT = L + 2 - (L & 1)
    max_len = int(rng.choice([L, L, int(rng.integers(1, L + 1)), 1024, 1025, 300]))
    T = rng.integers(0, 6 if rng.random() < 0.4 else 100000, size=(B, L, ldT)).astype(np.int64)
    T[rng.random(T.shape) < float(rng.choice([0, 0.05, 0.5]))] = INF
    masked = T.copy()
    i, j = np.meshgrid(np.arange(L), np.arange(ldT), indexing="ij")
    masked[:, j - i > max_len] = INF
    s_query = int(rng.integers(0, S + 1))
    want = oracle.stage_interval(masked, S, s_query=s_query, nthreads=8)
    bott = torch.full((B, S), -7, dtype=torch.int64, device=DEV)
    cut = torch.full((B, S, L + 1), -7, dtype=torch.int32, device=DEV)
    bounds = torch.full((B, s_query + 1), -7, dtype=torch.int32, device=DEV) if s_query else None
    ws = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP_INTERVAL, B, L, S), dtype=torch.uint8, device=DEV)
    if max_len >= L and rng.random() < 0.5:
        rh.rh_stage_dp_interval(B, L, S, ldT, torch.from_numpy(T).to(DEV), bott, cut, s_query, bounds, ws)
    else:
        rh.rh_stage_dp_interval_banded(B, L, S, min(max_len, L), ldT, torch.from_numpy(T).to(DEV), bott, cut, s_query,
                                       bounds, ws)
    torch.cuda.synchronize()
    assert np.array_equal(bott.cpu().numpy(), want[0]) and np.array_equal(cut.cpu().numpy(), want[1])
    if s_query:
        assert np.array_equal(bounds.cpu().numpy(), want[2])


def table_case(rng):
    Kp = int(rng.choice([16, 32, 64, 64, 64, 128, 256]))
    L = int(rng.integers(1, 900 if Kp == 64 else (200 if Kp < 256 else 60)))
    B = int(rng.integers(1, 4))
    K = int(rng.integers(max(1, Kp // 2), Kp + 1))
    ldT = L + 2 - (L & 1)
    c, R = rand_chain(rng, B, L, K, Kp, rng.random() < 0.3, float(rng.choice([0, 0.05])))
    mode = int(rng.integers(0, 3))                            # row by row, from blocks where the sizes allow, limited
    max_len = int(rng.integers(1, L + 1))
    dT = torch.full((B, L, ldT), -3, dtype=torch.int64, device=DEV)
    dc = torch.from_numpy(c).to(DEV)
    dR = torch.from_numpy(R).to(DEV) if L > 1 else None
    if mode == 2:
        need = rh.rh_workspace_size(rh.WS_INTERVAL_COSTS, B, L, Kp) if rng.random() < 0.5 else 0
        rh.rh_interval_costs_banded(B, L, Kp, max_len, dc, dR, ldT, dT,
                                    torch.empty(need, dtype=torch.uint8, device=DEV) if need else None)
    else:
        need = rh.rh_workspace_size(rh.WS_INTERVAL_COSTS, B, L, Kp) if mode == 1 else 0
        rh.rh_interval_costs(B, L, Kp, dc, dR, ldT, dT, torch.empty(need, dtype=torch.uint8, device=DEV) if need else None)
    torch.cuda.synchronize()
    got = dT.cpu().numpy()
    upper = np.zeros((L, ldT), bool)
    upper[np.triu_indices(L, 1, ldT)] = True                 # the entries the interface defines: i < j <= L
    upper[:, L + 1:] = False
    for p in range(B):
        want = oracle.interval_costs(np.ascontiguousarray(c[p]), np.ascontiguousarray(R[p]), ldT=ldT, nthreads=8,
                                     max_len=max_len if mode == 2 else 0)
        assert np.array_equal(got[p][upper], want[upper]), p


def plans_case(rng):
    Kp = int(rng.choice([16, 32, 64, 128, 256]))
    L = int(rng.integers(1, 500 if Kp <= 64 else 120))
    S = int(rng.integers(1, min(L, 40) + 1))
    B = int(rng.integers(1, 4))
    K = int(rng.integers(max(1, Kp // 2), Kp + 1))
    c, R = rand_chain(rng, B, L, K, Kp, rng.random() < 0.4, float(rng.choice([0, 0.1])))
    bounds = np.zeros((B, S + 1), np.int32)
    for p in range(B):
        cuts = np.sort(rng.choice(np.arange(1, L), size=S - 1, replace=False)) if S > 1 else np.zeros(0, np.int32)
        bounds[p] = np.concatenate([[0], cuts, [L]])
    if rng.random() < 0.2:
        bounds[0] = -1                                        # no split found for the first chain
    test_gpu_stage_plans.check(bounds, c, R)


def specs_case(rng):
    Kp = int(rng.choice([64, 128, 256]))
    N = int(rng.integers(2, 400 if Kp == 64 else (200 if Kp == 128 else 100)))
    words = rng.integers(0, 1 << 16, size=(2, N, Kp)).astype(np.uint32)
    ok = rng.random((2, N, Kp)) < float(rng.choice([0.5, 0.8, 1.0]))
    b0 = (words & 3) % 3 | (((words >> 2) & 3) << 2) | (((words >> 5) & 1) << 5)
    b1 = ((words >> 8) & 3) % 3 | (((words >> 10) & 3) << 2) | (((words >> 13) & 1) << 5)
    words = np.where(ok, (b0 | (b1 << 8)).astype(np.uint32), words)
    words[0, :, ::13] = sp.EMPTY
    dims = np.tile(np.array([[64, 128, 256, 512]], dtype=np.int64), (N - 1, 1))
    dims[::5] = [96, 64, 48, 1]                               # extents that some strides do not divide
    g = dict(K=rng.integers(Kp // 2, Kp + 1, size=N).astype(np.int32), out_spec=words[0], in_spec=words[1],
             dims=dims, elem_bytes=rng.choice([1, 2, 4], size=N - 1).astype(np.int32))
    known = [((4, 8), (12500, 150000), (5, 0)), ((32,), (50000,), (0,)), ((2, 2), (1000, 1000), (0, 3)),
             ((16, 4), (7, 9), (0, 0))]
    nb = int(rng.integers(1, 4))
    meshes = [known[int(rng.integers(0, 4))] for _ in range(nb)]
    cs = rng.integers(0, 100000, size=(nb, N, Kp)).astype(np.int64)
    cs[rng.random(cs.shape) < float(rng.choice([0, 0.3]))] = INF
    cs[:, :, 1] = 7                                           # one strategy stays in the game at every operator
    g["out_spec"][:, 1] = sp.word(sp.R_, sp.R_)
    seg = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SPECS, nb, N, Kp) > 0
    test_gpu_fused.check(g, meshes, cs, segmented=(False, True) if seg else (False,))


CASES = [chain_case, chain_case, tree_case, window_case, stage_case, search_case, table_case, specs_case, plans_case]


@pytest.mark.parametrize("seed", [11, 12, 13, 14])
def test_random_shapes(seed):
    rng = np.random.default_rng(seed)
    for k in range(60):
        case = CASES[int(rng.integers(0, len(CASES)))]
        state = rng.bit_generator.state
        try:
            case(rng)
        except AssertionError as e:
            raise AssertionError(f"case {k} ({case.__name__}) of seed {seed}; generator state before it: {state}") from e
