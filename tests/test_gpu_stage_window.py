"""GPU parity of the windowed pipeline-stage DP (transfers + bound tightening) against the CPU oracle."""
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


def gpu_window(cost, S, xfer, num, den):
    B, L = cost.shape
    bott = torch.full((B,), -7, dtype=torch.int64, device=DEV)
    cut = torch.full((B, S, L + 1), -7, dtype=torch.int32, device=DEV)
    bounds = torch.full((B, S + 1), -7, dtype=torch.int32, device=DEV)
    ws = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP_WINDOW, B, L, S), dtype=torch.uint8, device=DEV)
    rh.rh_stage_dp_window(B, L, S, torch.from_numpy(cost).to(DEV),
                          torch.from_numpy(xfer).to(DEV) if xfer is not None else None, num, den, bott, cut, bounds, ws)
    torch.cuda.synchronize()
    return bott.cpu().numpy(), cut.cpu().numpy(), bounds.cpu().numpy()


def check(cost, S, xfer, num, den):
    want = oracle.stage_window(cost, S, xfer, num, den)
    got = gpu_window(cost, S, xfer, num, den)
    assert np.array_equal(got[0], want[0]), (num, den)
    assert np.array_equal(got[1], want[1]), (num, den)
    assert np.array_equal(got[2], want[2]), (num, den)
    return want[0]


@pytest.mark.parametrize("L,S,B", [(1, 1, 1), (7, 3, 2), (64, 8, 2), (65, 5, 3), (200, 16, 2), (1000, 64, 2)])
def test_shapes_and_tolerances(L, S, B):
    rng = np.random.default_rng(L * 31 + S)
    cost = np.stack([syn.segment_costs(p, L) for p in range(B)])
    xfer = rng.integers(0, 20000, size=(B, L + 1)).astype(np.int64)
    for num, den in ((-1, 1), (0, 1), (1, 8), (1, 2), (1, 1), (5, 2)):
        check(cost, S, xfer, num, den)
    check(cost, S, None, 1, 4)


def test_ties_zero_costs_and_no_split():
    rng = np.random.default_rng(5)
    cost = rng.integers(0, 3, size=(3, 150)).astype(np.int64)
    cost[1] = 0                                              # total 0: the bounds are switched off
    cost[2, :75] = 0                                         # all the work in the second half
    xfer = rng.integers(0, 3, size=(3, 151)).astype(np.int64)
    for num, den in ((0, 1), (1, 3), (2, 1)):
        b = check(cost, 12, xfer, num, den)
    # one huge segment: with a tight tolerance no split into many stages exists
    spike = np.ones((1, 40), dtype=np.int64)
    spike[0, 20] = 10**6
    b = check(spike, 8, None, 0, 1)
    assert b[0] == INF
    assert check(spike, 8, None, 10, 1)[0] < INF


def test_segments_of_very_different_size():
    # thousands of cheap segments between a few heavy ones: whatever the tolerance suggests about the width of
    # a stage count's window, a tile's rows here run into the thousands
    rng = np.random.default_rng(17)
    L, S = 5000, 16
    cost = rng.integers(0, 3, size=(2, L)).astype(np.int64)
    heavy = rng.choice(L, size=40, replace=False)
    cost[0, heavy] = rng.integers(10**5, 10**6, size=40)
    cost[1, heavy[:9]] = 10**6
    xfer = rng.integers(0, 5000, size=(2, L + 1)).astype(np.int64)
    for num, den in ((1, 2), (3, 1), (-1, 1)):
        check(cost, S, xfer, num, den)


def test_stage_partition_config_full_size_window():
    w = syn.STAGE_PARTITION
    cost = syn.segment_costs(0, w["L"], w["lo"], w["hi"])[None]
    xfer = syn.uniform_at(syn.stream_seed(syn.BASE_SEED, 0, 7), np.arange(w["L"] + 1, dtype=np.uint64), 50000)[None]
    plain = oracle.stage_dp(cost, w["S"])[0][0, w["S"] - 1]
    b = check(cost, w["S"], np.ascontiguousarray(xfer), 1, 2)
    assert b[0] >= plain
    assert check(cost, w["S"], None, -1, 1)[0] == plain


def test_argument_errors():
    L = rh.lib()
    t = torch.zeros(4096, dtype=torch.int64, device=DEV)
    P = ctypes.c_void_p(t.data_ptr())
    ws = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP_WINDOW, 1, 64, 8), dtype=torch.uint8, device=DEV)
    W = ctypes.c_void_p(ws.data_ptr())
    call = lambda S=8, den=1, wsb=ws.numel(), cost=P: L.rh_stage_dp_window(1, 64, S, cost, None, 1, den, P, P, None,
                                                                         W, wsb, None)
    assert call(S=65) == -2 and call(den=0) == -2 and call(cost=None) == -1 and call(wsb=64) == -4
    assert rh.rh_workspace_size(rh.WS_STAGE_DP_WINDOW, 1, 64, 8) > rh.rh_workspace_size(rh.WS_STAGE_DP, 1, 64, 8)
    torch.cuda.synchronize()
