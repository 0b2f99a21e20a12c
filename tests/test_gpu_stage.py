"""GPU parity of the pipeline-stage DP against the CPU oracle (bit-exact)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import synthetic as syn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def gpu_stage(cost, S, s_query):
    B, L = cost.shape
    d_cost = torch.from_numpy(cost).to(DEV)
    bott = torch.full((B, S), -7, dtype=torch.int64, device=DEV)
    cut = torch.full((B, S, L + 1), -7, dtype=torch.int32, device=DEV)
    bounds = torch.full((B, s_query + 1), -7, dtype=torch.int32, device=DEV) if s_query else None
    ws = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP, B, L, S), dtype=torch.uint8, device=DEV)
    rh.rh_stage_dp(B, L, S, d_cost, bott, cut, s_query, bounds, ws)
    torch.cuda.synchronize()
    return bott.cpu().numpy(), cut.cpu().numpy(), bounds.cpu().numpy() if s_query else None


def check(cost, S, s_query):
    o_b, o_c, o_bd = oracle.stage_dp(cost, S, s_query=s_query, nthreads=4)
    g_b, g_c, g_bd = gpu_stage(cost, S, s_query)
    assert np.array_equal(g_b, o_b)
    assert np.array_equal(g_c, o_c)
    if s_query:
        assert np.array_equal(g_bd, o_bd)


@pytest.mark.parametrize("L,S,B", [(1, 1, 1), (5, 5, 3), (63, 7, 2), (64, 64, 2), (65, 16, 2), (200, 33, 3),
                                    (1000, 64, 2), (4096, 8, 1)])
def test_shapes_around_the_tile_size(L, S, B):
    cost = np.stack([syn.segment_costs(p, L) for p in range(B)])
    check(cost, S, s_query=min(S, 5))


def test_many_ties():
    rng = np.random.default_rng(0)
    cost = rng.integers(1, 3, size=(4, 300)).astype(np.int64)
    check(cost, 40, s_query=40)
    check(np.full((1, 257), 9, dtype=np.int64), 64, s_query=64)
    check(np.zeros((1, 130), dtype=np.int64), 9, s_query=9)           # zero costs are allowed


def test_stage_partition_config_full_size():
    w = syn.STAGE_PARTITION
    cost = syn.segment_costs(0, w["L"], w["lo"], w["hi"])[None]
    check(cost, w["S"], s_query=w["S"])


def test_argument_errors():
    L = rh.lib()
    t = torch.zeros(4096, dtype=torch.int64, device=DEV)
    P = lambda x: ctypes.c_void_p(x.data_ptr())
    ws = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP, 1, 64, 8), dtype=torch.uint8, device=DEV)
    ok = lambda **kw: L.rh_stage_dp(kw.get("B", 1), kw.get("L", 64), kw.get("S", 8), P(t), P(t), P(t),
                                    kw.get("sq", 0), None, kw.get("ws", P(ws)), kw.get("wsb", ws.numel()), None)
    assert ok(S=65) == -2 and ok(L=0) == -2 and ok(S=0) == -2 and ok(sq=9) == -2
    assert ok(sq=3) == -1                                             # bounds wanted but NULL
    assert ok(ws=None) == -4 and ok(wsb=16) == -4
    assert rh.rh_workspace_size(rh.WS_STAGE_DP, 1, 64, 65) == 0
    torch.cuda.synchronize()


@pytest.mark.parametrize("L,S,B", [(6143, 6, 1), (6144, 6, 1), (6209, 5, 2), (8191, 3, 1)])
def test_both_sides_of_the_lds_limit(L, S, B):
    # up to 6143 segments one workgroup bisects in LDS; longer chains scan every (i, j) cell
    cost = np.stack([syn.segment_costs(p, L) for p in range(B)])
    check(cost, S, s_query=S)


def test_many_ties_on_long_chains():
    rng = np.random.default_rng(5)
    cost = rng.integers(0, 3, size=(2, 6300)).astype(np.int64)        # plateaus of zero-cost segments
    check(cost, 7, s_query=7)
    cost = (rng.integers(0, 2, size=(1, 6100)) * rng.integers(0, 4, size=(1, 6100))).astype(np.int64)
    check(cost, 33, s_query=33)


def test_long_chain_of_segments():
    # beyond one split's worth of i per workgroup and beyond 2^16 / 4 segments
    cost = syn.segment_costs(3, 20000)[None]
    check(cost, 6, s_query=6)
