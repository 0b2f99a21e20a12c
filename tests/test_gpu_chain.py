"""GPU parity of the chain DP and backtrack against the CPU oracle (bit-exact)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import device_fill, synthetic as syn

pytestmark = pytest.mark.gpu
INF = oracle.INF
DEV = "cuda:0"


def gpu_chain(c, R, shared_R=False, want_vfinal=True):
    B, N, Kp = c.shape
    dc = torch.from_numpy(c).to(DEV)
    dR = torch.from_numpy(R).to(DEV) if R.size else None
    arg = torch.full((B, max(N - 1, 0), Kp), -1, dtype=torch.int16, device=DEV)
    vfinal = torch.zeros((B, Kp), dtype=torch.int64, device=DEV) if want_vfinal else None
    total = torch.zeros(B, dtype=torch.int64, device=DEV)
    last = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    plan = torch.full((B, N), -1, dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain(B, N, Kp, dc, N * Kp, dR, 0 if shared_R else (N - 1) * Kp * Kp, arg if N > 1 else None,
                        vfinal, total, last)
    rh.rh_backtrack(B, N, Kp, arg if N > 1 else None, last, plan)
    torch.cuda.synchronize()
    return (arg.cpu().numpy().view(np.uint16), vfinal.cpu().numpy() if want_vfinal else None,
            total.cpu().numpy(), last.cpu().numpy(), plan.cpu().numpy())


def check(c, R, shared_R=False):
    o_arg, o_vf, o_total, o_last = oracle.chain(c, R, nthreads=4, shared_R=shared_R)
    o_plan = oracle.backtrack(o_arg, o_last)
    g_arg, g_vf, g_total, g_last, g_plan = gpu_chain(c, R, shared_R)
    assert np.array_equal(g_total, o_total)
    assert np.array_equal(g_last, o_last)
    assert np.array_equal(g_vf, o_vf)
    assert np.array_equal(g_arg, o_arg)
    assert np.array_equal(g_plan, o_plan)


def test_tiny_chain_config():
    w = syn.TINY_CHAIN
    c, R = syn.random_chain_batch([0], w["N"], w["K"], w["c_range"], w["r_range"], Kp=16)
    check(c, R)


@pytest.mark.parametrize("Kp", [16, 32, 64, 128, 256, 512, 1024])
def test_every_tile_width(Kp):
    # several edges per problem, a ragged number of problems per workgroup, full and padded K
    B, N = (7, 5) if Kp <= 256 else (3, 3)
    K = Kp if Kp % 32 == 0 and Kp != 64 else Kp - 3
    c, R = syn.random_chain_batch(range(B), N, K, 1000, 5000, Kp=Kp)
    check(c, R)


@pytest.mark.parametrize("Kp,N", [(16, 4), (32, 4), (64, 4), (128, 3), (256, 3), (512, 2), (1024, 2)])
def test_many_problems_one_wave_each(Kp, N):
    # 2048 problems and more run one wavefront per problem; fewer run a workgroup per problem
    B = 2048 + 3
    c = torch.empty((B, N, Kp), dtype=torch.int64, device=DEV)
    R = torch.empty((B, N - 1, Kp, Kp), dtype=torch.int64, device=DEV)
    device_fill.fill_random_chain(c, R, 5000, 1000, 5000)
    arg = torch.full((B, N - 1, Kp), -1, dtype=torch.int16, device=DEV)
    vfinal = torch.zeros((B, Kp), dtype=torch.int64, device=DEV)
    total = torch.zeros(B, dtype=torch.int64, device=DEV)
    last = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    plan = torch.full((B, N), -1, dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain(B, N, Kp, c, N * Kp, R, (N - 1) * Kp * Kp, arg, vfinal, total, last)
    rh.rh_backtrack(B, N, Kp, arg, last, plan)
    torch.cuda.synchronize()
    sel = list(range(B)) if Kp <= 128 else [0, 1, 2, 3, 64, 999, 2047, 2048, 2049, 2050]
    idx = torch.tensor(sel, device=DEV)
    o_arg, o_vf, o_total, o_last = oracle.chain(c[idx].cpu().numpy(), R[idx].cpu().numpy(), nthreads=8)
    assert np.array_equal(total[idx].cpu().numpy(), o_total) and np.array_equal(last[idx].cpu().numpy(), o_last)
    assert np.array_equal(vfinal[idx].cpu().numpy(), o_vf)
    assert np.array_equal(arg[idx].cpu().numpy().view(np.uint16), o_arg)
    assert np.array_equal(plan[idx].cpu().numpy(), oracle.backtrack(o_arg, o_last))


@pytest.mark.parametrize("Kp,N,B", [(128, 40, 9), (64, 33, 13), (256, 9, 5), (128, 6, 700), (256, 5, 600),
                                     (32, 9, 100), (512, 4, 3), (1024, 3, 2)])
def test_longer_chains(Kp, N, B):
    c, R = syn.random_chain_batch(range(100, 100 + B), N, Kp, 1_000_000, 10_000_000, Kp=Kp)
    check(c, R)


@pytest.mark.parametrize("Kp,N,B", [(256, 64, 1), (256, 131, 3), (128, 64, 2), (128, 257, 32), (256, 70, 32),
                                    (256, 70, 33), (256, 64, 40), (128, 80, 50), (128, 64, 64)])
def test_few_long_chains_spread_over_several_workgroups(Kp, N, B):
    # with a workspace, few long chains of wide tables run eight workgroups per problem, four when there are more
    # than 32 problems
    need = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, B, N, Kp)
    assert need > 0
    rng = np.random.default_rng(B * 1000 + N)
    c, R = syn.random_chain_batch(range(40, 40 + B), N, Kp, 1_000_000, 10_000_000)
    if B > 1:
        # problem 1: ties everywhere and infeasible entries
        c[1] = rng.integers(0, 3, size=c[1].shape)
        R[1] = rng.integers(0, 3, size=R[1].shape)
        R[1][rng.random(R[1].shape) < 0.4] = INF
        c[1, N // 2, Kp // 3:] = INF
    if B > 2:
        c[2, N // 3, :] = INF                                         # nothing feasible from there on
    # empty candidate slots: whole rows and columns of R are infeasible, as in tables built from specs
    c[0, :, Kp - 37:] = INF
    R[0, :, Kp - 37:, :] = INF
    R[0, :, :, Kp - 37:] = INF
    o_arg, o_vf, o_total, o_last = oracle.chain(c, R, nthreads=8)
    dc, dR = torch.from_numpy(c).to(DEV), torch.from_numpy(R).to(DEV)
    for use_ws in (True, False, True):
        arg = torch.full((B, N - 1, Kp), -1, dtype=torch.int16, device=DEV)
        vfinal = torch.zeros((B, Kp), dtype=torch.int64, device=DEV)
        total = torch.zeros(B, dtype=torch.int64, device=DEV)
        last = torch.full((B,), -1, dtype=torch.int32, device=DEV)
        ws = torch.full((need,), 0xAB, dtype=torch.uint8, device=DEV) if use_ws else None   # stale contents
        rh.rh_minplus_chain(B, N, Kp, dc, N * Kp, dR, (N - 1) * Kp * Kp, arg, vfinal, total, last, ws)
        torch.cuda.synchronize()
        assert np.array_equal(total.cpu().numpy(), o_total), use_ws
        assert np.array_equal(last.cpu().numpy(), o_last)
        assert np.array_equal(vfinal.cpu().numpy(), o_vf)
        assert np.array_equal(arg.cpu().numpy().view(np.uint16), o_arg)
    # too many problems to keep every gang resident
    assert rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, 65, N, Kp) == 0
    assert rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, B, 63, Kp) == 0 and rh.rh_workspace_size(0, B, N, 64) == 0


@pytest.mark.parametrize("Kp,N,B", [(64, 512, 1), (64, 1000, 2), (128, 777, 1), (256, 600, 2), (256, 1153, 1),
                                    (64, 128, 1), (64, 243, 2), (128, 200, 1), (256, 129, 2)])
def test_one_long_chain_cut_into_segments(Kp, N, B):
    # with a workspace, one or two long chains are solved segment by segment (matrices, boundary vectors, batch)
    need = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, B, N, Kp)
    assert need > 0
    assert rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, B, 127, 64) == 0
    rng = np.random.default_rng(Kp + N)
    K = Kp - (Kp // 5 if N % 2 else 0)                                # some shapes with empty candidate slots
    c, R = syn.random_chain_batch(range(60, 60 + B), N, K, 1_000_000, 10_000_000, Kp=Kp)
    # infeasible strategies scattered over the operators (as in tables built from specs)
    dead = rng.random((B, N, Kp)) < 0.3
    dead[:, :, 0] = False
    c[dead] = INF
    if B > 1:
        # problem 1: ties everywhere and infeasible pairs
        c[1] = rng.integers(0, 3, size=c[1].shape)
        R[1] = rng.integers(0, 3, size=R[1].shape)
        R[1][rng.random(R[1].shape) < 0.4] = INF
        c[1, N // 2, Kp // 3:] = INF
    o_arg, o_vf, o_total, o_last = oracle.chain(c, R, nthreads=8)
    dc, dR = torch.from_numpy(c).to(DEV), torch.from_numpy(R).to(DEV)
    for use_ws in (True, False, True):
        arg = torch.full((B, N - 1, Kp), -1, dtype=torch.int16, device=DEV)
        vfinal = torch.zeros((B, Kp), dtype=torch.int64, device=DEV)
        total = torch.zeros(B, dtype=torch.int64, device=DEV)
        last = torch.full((B,), -1, dtype=torch.int32, device=DEV)
        ws = torch.full((need,), 0xAB, dtype=torch.uint8, device=DEV) if use_ws else None   # stale contents
        rh.rh_minplus_chain(B, N, Kp, dc, N * Kp, dR, (N - 1) * Kp * Kp, arg, vfinal, total, last, ws)
        torch.cuda.synchronize()
        assert np.array_equal(total.cpu().numpy(), o_total), use_ws
        assert np.array_equal(last.cpu().numpy(), o_last)
        assert np.array_equal(vfinal.cpu().numpy(), o_vf)
        assert np.array_equal(arg.cpu().numpy().view(np.uint16), o_arg)


@pytest.mark.parametrize("Kp,N,B", [(64, 273, 1), (64, 2000, 3), (128, 529, 16), (256, 1041, 2), (256, 8192, 1),
                                    (1024, 16384, 1), (512, 5000, 2), (64, 272, 1), (128, 3000, 17)])
def test_backtrack_of_long_chains(Kp, N, B):
    # a few long chains are walked in blocks of rows (maps per block, composed, then every block walked); any
    # table of row indices will do, also one that never came from a sweep
    rng = np.random.default_rng(Kp * 7 + N)
    arg = rng.integers(0, Kp, size=(B, N - 1, Kp)).astype(np.uint16)
    if B > 1:
        arg[1] = (np.arange(Kp, dtype=np.uint16) * 5 + 3) % Kp        # the same permutation in every row
    last = rng.integers(0, Kp, size=B).astype(np.int32)
    want = oracle.backtrack(arg, last)
    d_arg = torch.from_numpy(arg.view(np.int16)).to(DEV)
    d_last = torch.from_numpy(last).to(DEV)
    for fill in (-1, 7):                                              # whatever the plan buffer held before
        plan = torch.full((B, N), fill, dtype=torch.int32, device=DEV)
        rh.rh_backtrack(B, N, Kp, d_arg, d_last, plan)
        torch.cuda.synchronize()
        assert np.array_equal(plan.cpu().numpy(), want)


@pytest.mark.parametrize("Kp,N", [(64, 900), (256, 700)])
def test_segmented_chain_with_awkward_feasibility(Kp, N):
    # feasible sets that change from operator to operator: alternating halves, single survivors, a first operator
    # with one feasible strategy, and edge tables with whole infeasible blocks
    rng = np.random.default_rng(Kp + 1)
    B = 2
    c = rng.integers(0, 1000, size=(B, N, Kp)).astype(np.int64)
    R = rng.integers(0, 1000, size=(B, N - 1, Kp, Kp)).astype(np.int64)
    half = np.arange(Kp) % 2
    for i in range(N):
        c[0, i, half == (i % 2)] = INF                                # even operators keep odd slots and vice versa
    for i in range(0, N, 37):
        keep = int(rng.integers(0, Kp // 2)) * 2 + (1 - i % 2)        # one survivor, of the right parity
        c[0, i, :] = INF
        c[0, i, keep] = int(rng.integers(0, 1000))
    c[1, :, Kp // 4:] = INF                                           # a quarter of the slots in use
    R[1, :, : Kp // 8, Kp // 8: Kp // 4] = INF                        # a block nobody can cross
    R[1, 100:, Kp // 8: Kp // 4, : Kp // 8] = INF
    o_arg, o_vf, o_total, o_last = oracle.chain(c, R, nthreads=8)
    assert o_total[0] < INF and o_total[1] < INF
    dc, dR = torch.from_numpy(c).to(DEV), torch.from_numpy(R).to(DEV)
    need = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, B, N, Kp)
    assert need > 0
    ws = torch.full((need,), 0x5A, dtype=torch.uint8, device=DEV)
    arg = torch.full((B, N - 1, Kp), -1, dtype=torch.int16, device=DEV)
    vfinal = torch.zeros((B, Kp), dtype=torch.int64, device=DEV)
    total = torch.zeros(B, dtype=torch.int64, device=DEV)
    last = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain(B, N, Kp, dc, N * Kp, dR, (N - 1) * Kp * Kp, arg, vfinal, total, last, ws)
    torch.cuda.synchronize()
    assert np.array_equal(total.cpu().numpy(), o_total) and np.array_equal(last.cpu().numpy(), o_last)
    assert np.array_equal(vfinal.cpu().numpy(), o_vf)
    assert np.array_equal(arg.cpu().numpy().view(np.uint16), o_arg)


@pytest.mark.parametrize("Kp,N,live", [(128, 400, 20), (256, 500, 150), (256, 300, 33), (128, 700, 100)])
def test_segmented_chain_by_number_of_feasible_strategies(Kp, N, live):
    # the kernels of the segmented path size their loops by the number of feasible strategies (rows in flight per
    # wave, width of the staged tables): few, just past a power of two, and most of them
    rng = np.random.default_rng(Kp + live)
    c = rng.integers(0, 1000, size=(1, N, Kp)).astype(np.int64)
    R = rng.integers(0, 1000, size=(1, N - 1, Kp, Kp)).astype(np.int64)
    for i in range(N):
        n_i = live if i % 7 else max(1, live // 3)                    # every seventh operator is narrow
        dead = rng.permutation(Kp)[n_i:]
        c[0, i, dead] = INF
    R[0][rng.random(size=(N - 1, Kp, Kp)) < 0.05] = INF               # and some pairs cannot be converted
    o_arg, o_vf, o_total, o_last = oracle.chain(c, R, nthreads=8)
    dc, dR = torch.from_numpy(c).to(DEV), torch.from_numpy(R).to(DEV)
    need = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, 1, N, Kp)
    assert need > 0
    ws = torch.full((need,), 0xA5, dtype=torch.uint8, device=DEV)
    arg = torch.full((1, N - 1, Kp), -1, dtype=torch.int16, device=DEV)
    vfinal = torch.zeros((1, Kp), dtype=torch.int64, device=DEV)
    total = torch.zeros(1, dtype=torch.int64, device=DEV)
    last = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain(1, N, Kp, dc, N * Kp, dR, (N - 1) * Kp * Kp, arg, vfinal, total, last, ws)
    torch.cuda.synchronize()
    assert np.array_equal(total.cpu().numpy(), o_total) and np.array_equal(last.cpu().numpy(), o_last)
    assert np.array_equal(vfinal.cpu().numpy(), o_vf)
    assert np.array_equal(arg.cpu().numpy().view(np.uint16), o_arg)


def test_several_chains_through_the_segmented_route():
    # more than two problems take the segmented route when the caller brings its workspace; R shared or not
    rng = np.random.default_rng(77)
    B, N, Kp = 5, 300, 128
    c = rng.integers(0, 1000, size=(B, N, Kp)).astype(np.int64)
    c[rng.random(size=c.shape) < 0.6] = INF
    c[:, :, 0] = rng.integers(0, 1000, size=(B, N))                   # strategy 0 stays feasible everywhere
    for shared in (False, True):
        R = rng.integers(0, 1000, size=(1 if shared else B, N - 1, Kp, Kp)).astype(np.int64)
        o_arg, o_vf, o_total, o_last = (oracle.chain(c, R[0], nthreads=8, shared_R=True) if shared
                                        else oracle.chain(c, R, nthreads=8))
        dc, dR = torch.from_numpy(c).to(DEV), torch.from_numpy(R).to(DEV)
        need = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SEGMENTED, B, N, Kp)
        assert need > rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, B, N, Kp) > 0
        # only the exact size asks for the segmented route; a larger pool takes the default route of these sizes
        # (same results either way)
        ws = torch.empty(need if shared else need + 4096, dtype=torch.uint8, device=DEV)
        arg = torch.full((B, N - 1, Kp), -1, dtype=torch.int16, device=DEV)
        vfinal = torch.zeros((B, Kp), dtype=torch.int64, device=DEV)
        total = torch.zeros(B, dtype=torch.int64, device=DEV)
        last = torch.full((B,), -1, dtype=torch.int32, device=DEV)
        rh.rh_minplus_chain(B, N, Kp, dc, N * Kp, dR, 0 if shared else (N - 1) * Kp * Kp, arg, vfinal, total, last, ws)
        torch.cuda.synchronize()
        assert np.array_equal(total.cpu().numpy(), o_total) and np.array_equal(last.cpu().numpy(), o_last)
        assert np.array_equal(vfinal.cpu().numpy(), o_vf)
        assert np.array_equal(arg.cpu().numpy().view(np.uint16), o_arg)


@pytest.mark.parametrize("seed", range(10))
def test_segmented_chain_on_random_shapes_and_feasible_sets(seed):
    # shapes, batch sizes and feasibility patterns drawn at random: every operator gets its own share of feasible
    # strategies (now and then a single one, now and then all), some pairs cannot be converted, ties are common
    rng = np.random.default_rng(1000 + seed)
    Kp = int(rng.choice([64, 128, 256]))
    N = int(rng.integers(128, 420))
    B = int(rng.integers(1, 4))
    c = rng.integers(0, 40, size=(B, N, Kp)).astype(np.int64)
    R = rng.integers(0, 40, size=(B, N - 1, Kp, Kp)).astype(np.int64)
    for p in range(B):
        for i in range(N):
            share = rng.choice([1.0 / Kp, 0.1, 0.3, 0.6, 1.0], p=[0.05, 0.2, 0.4, 0.25, 0.1])
            keep = rng.random(Kp) < share
            keep[int(rng.integers(0, Kp))] = True
            c[p, i, ~keep] = INF
    R[rng.random(size=R.shape) < 0.02] = INF
    o_arg, o_vf, o_total, o_last = oracle.chain(c, R, nthreads=8)
    dc, dR = torch.from_numpy(c).to(DEV), torch.from_numpy(R).to(DEV)
    need = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SEGMENTED, B, N, Kp)
    assert need > 0
    ws = torch.full((need,), 0x3C, dtype=torch.uint8, device=DEV)
    arg = torch.full((B, N - 1, Kp), -1, dtype=torch.int16, device=DEV)
    vfinal = torch.zeros((B, Kp), dtype=torch.int64, device=DEV)
    total = torch.zeros(B, dtype=torch.int64, device=DEV)
    last = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain(B, N, Kp, dc, N * Kp, dR, (N - 1) * Kp * Kp, arg, vfinal, total, last, ws)
    torch.cuda.synchronize()
    assert np.array_equal(total.cpu().numpy(), o_total) and np.array_equal(last.cpu().numpy(), o_last)
    assert np.array_equal(vfinal.cpu().numpy(), o_vf)
    assert np.array_equal(arg.cpu().numpy().view(np.uint16), o_arg)


def test_long_chain_that_dies_in_the_middle():
    # nothing is feasible from one operator on: every later segment starts from an all-infeasible vector
    Kp, N = 64, 700
    c, R = syn.random_chain_batch([9], N, Kp, 1000, 5000)
    c[0, 300, :] = INF
    o_arg, o_vf, o_total, o_last = oracle.chain(c, R)
    dc, dR = torch.from_numpy(c).to(DEV), torch.from_numpy(R).to(DEV)
    ws = torch.empty(rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, 1, N, Kp), dtype=torch.uint8, device=DEV)
    arg = torch.full((1, N - 1, Kp), -1, dtype=torch.int16, device=DEV)
    vfinal = torch.zeros((1, Kp), dtype=torch.int64, device=DEV)
    total = torch.zeros(1, dtype=torch.int64, device=DEV)
    last = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain(1, N, Kp, dc, N * Kp, dR, (N - 1) * Kp * Kp, arg, vfinal, total, last, ws)
    torch.cuda.synchronize()
    assert total.item() == INF == o_total[0] and last.item() == o_last[0]
    assert np.array_equal(vfinal.cpu().numpy(), o_vf)
    assert np.array_equal(arg.cpu().numpy().view(np.uint16), o_arg)


@pytest.mark.parametrize("Kp", [16, 64, 128])
def test_ties_ragged_and_infeasible(Kp):
    rng = np.random.default_rng(Kp)
    B, N = 6, 7
    c = rng.integers(0, 3, size=(B, N, Kp)).astype(np.int64)          # {0,1,2}: ties everywhere
    R = rng.integers(0, 3, size=(B, N - 1, Kp, Kp)).astype(np.int64)
    for p in range(B):
        Ki = rng.integers(1, Kp + 1, size=N)
        for i in range(N):
            c[p, i, Ki[i]:] = INF
            if i < N - 1:
                R[p, i, Ki[i]:, :] = INF
            if i > 0:
                R[p, i - 1, :, Ki[i]:] = INF
    R[1][rng.random(R[1].shape) < 0.5] = INF
    c[2, 3, :] = INF                                                  # problem 2 has no feasible plan
    check(c, R)
    _, _, total, last, plan = gpu_chain(c, R)
    assert total[2] == INF and last[2] == 0 and not plan[2, 3:].any()   # nothing feasible from operator 3 on


def test_shared_R_single_operator_and_empty_batch():
    c, R = syn.random_chain_batch(range(4), 6, 64, 1000, 5000)
    check(c, np.ascontiguousarray(R[0]), shared_R=True)
    c1 = c[:, :1].copy()                                              # N = 1: total = min c_0
    _, vf, total, last, plan = gpu_chain(c1, np.zeros((4, 0, 64, 64), np.int64))
    assert np.array_equal(total, c1[:, 0].min(axis=1)) and np.array_equal(last, c1[:, 0].argmin(axis=1))
    assert np.array_equal(plan[:, 0], last) and np.array_equal(vf, c1[:, 0])
    e = torch.empty(0, dtype=torch.int64, device=DEV)
    rh.rh_minplus_chain(0, 5, 64, e, 0, e, 0, None, None, e, torch.empty(0, dtype=torch.int32, device=DEV))


def test_argument_errors_launch_nothing():
    # straight through the C ABI: the checks run on the host before any launch
    import ctypes
    L = rh.lib()
    t64 = torch.zeros(64 * 64 * 2, dtype=torch.int64, device=DEV)
    t32 = torch.zeros(64, dtype=torch.int32, device=DEV)
    t16 = torch.zeros(64 * 2, dtype=torch.int16, device=DEV)
    P = lambda t, off=0: ctypes.c_void_p(t.data_ptr() + off)

    def call(B=1, N=2, Kp=64, c=P(t64), R=P(t64), total=P(t64)):
        return L.rh_minplus_chain(B, N, Kp, c, 128, R, 4096, P(t16), None, total, P(t32), None, 0, None)

    assert call() == 0
    assert call(Kp=48) == -3 and call(Kp=8) == -3 and call(Kp=2048) == -3
    assert call(N=0) == -2 and call(N=20000) == -2 and call(B=-1) == -2
    assert call(c=None) == -1 and call(R=None) == -1 and call(total=None) == -1
    assert call(c=P(t64, 8)) == -2                                    # rows not 16-byte aligned
    assert L.rh_backtrack(1, 2, 63, P(t16), P(t32), P(t32), None) == -3
    assert L.rh_backtrack(1, 2, 64, P(t16), None, P(t32), None) == -1
    torch.cuda.synchronize()
    assert "power of two" in rh.strerror(-3)
    # the binding refuses buffers shorter than the sizes say
    with pytest.raises(ValueError):
        rh.rh_minplus_chain(4, 2, 64, t64[:256], 128, t64, 4096, t16, None, t64, t32)


def test_device_fill_matches_host_generator():
    B, N, K = 5, 4, 64
    c = torch.empty((B, N, K), dtype=torch.int64, device=DEV)
    R = torch.empty((B, N - 1, K, K), dtype=torch.int64, device=DEV)
    device_fill.fill_random_chain(c, R, first_problem=37, c_range=1_000_000, r_range=10_000_000)
    hc, hR = syn.random_chain_batch(range(37, 37 + B), N, K, 1_000_000, 10_000_000)
    assert np.array_equal(c.cpu().numpy(), hc) and np.array_equal(R.cpu().numpy(), hR)


def test_check_costs_counts_contract_violations():
    x = torch.tensor([0, 5, INF, (1 << 36) - 1, 1 << 36, -1, INF + 1], dtype=torch.int64, device=DEV)
    bad = torch.zeros(1, dtype=torch.int64, device=DEV)
    rh.rh_check_costs(x, bad)
    torch.cuda.synchronize()
    assert bad.item() == 3


@pytest.mark.parametrize("Kp,B", [(16, 3), (128, 1)])
def test_longest_chain_the_interface_allows(Kp, B):
    N = 16384
    rng = np.random.default_rng(Kp)
    c = rng.integers(0, 1 << 20, size=(B, N, Kp)).astype(np.int64)
    R = rng.integers(0, 1 << 20, size=(B, N - 1, Kp, Kp)).astype(np.int64)
    check(c, R)
    if Kp == 128:                                                     # and cut into segments
        dc, dR = torch.from_numpy(c).to(DEV), torch.from_numpy(R).to(DEV)
        ws = torch.empty(rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, B, N, Kp), dtype=torch.uint8, device=DEV)
        total = torch.zeros(B, dtype=torch.int64, device=DEV)
        last = torch.zeros(B, dtype=torch.int32, device=DEV)
        arg = torch.zeros((B, N - 1, Kp), dtype=torch.int16, device=DEV)
        rh.rh_minplus_chain(B, N, Kp, dc, N * Kp, dR, (N - 1) * Kp * Kp, arg, None, total, last, ws)
        torch.cuda.synchronize()
        o_arg, _, o_total, o_last = oracle.chain(c, R)
        assert total.item() == o_total[0] and np.array_equal(arg.cpu().numpy().view(np.uint16), o_arg)
