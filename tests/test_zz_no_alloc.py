"""rh_stage_dp_window_static (the entry point that allocates nothing) against rh_stage_dp_window, through the C ABI."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import synthetic as syn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def both(B, L, S, seed, num, den, fill):
    """One problem batch through both entry points, called straight through ctypes with raw pointers."""
    lib = rh.lib()
    rng = np.random.default_rng(seed)
    cost = torch.from_numpy(np.stack([syn.segment_costs(seed + p, L) for p in range(B)])).to(DEV)
    xfer = torch.from_numpy(rng.integers(0, 30000, size=(B, L + 1)).astype(np.int64)).to(DEV)
    P = lambda t: ctypes.c_void_p(t.data_ptr())
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    out = []
    for static in (False, True):
        bott = torch.full((B,), fill, dtype=torch.int64, device=DEV)
        cut = torch.full((B, S, L + 1), fill, dtype=torch.int32, device=DEV)
        bounds = torch.full((B, S + 1), fill, dtype=torch.int32, device=DEV)
        if static:
            rc = lib.rh_stage_dp_window_static(B, L, S, P(cost), P(xfer), num, den, P(bott), P(cut), P(bounds), stream)
        else:
            ws = torch.full((rh.rh_workspace_size(rh.WS_STAGE_DP_WINDOW, B, L, S),), 0x77, dtype=torch.uint8,
                            device=DEV)
            rc = lib.rh_stage_dp_window(B, L, S, P(cost), P(xfer), num, den, P(bott), P(cut), P(bounds), P(ws),
                                        ws.numel(), stream)
        assert rc == 0, rh.strerror(rc)
        torch.cuda.synchronize()
        out.append((bott.cpu().numpy(), cut.cpu().numpy(), bounds.cpu().numpy()))
    want = oracle.stage_window(cost.cpu().numpy(), S, xfer.cpu().numpy(), num, den)
    for a, b, o in zip(out[0], out[1], want):
        assert np.array_equal(a, b)
        assert np.array_equal(b, o)
    return out[1][0]


def test_two_calls_in_a_row_the_second_smaller():
    # the second call finds the first one's leftovers in the shared scratch
    big = both(3, 2500, 48, seed=100, num=1, den=2, fill=-7)
    small = both(2, 333, 9, seed=200, num=1, den=4, fill=-9)
    again = both(3, 2500, 48, seed=100, num=1, den=2, fill=-3)
    assert (big > 0).all() and (small > 0).all() and np.array_equal(big, again)


def test_sizes_beyond_the_static_scratch_are_refused():
    lib = rh.lib()
    cap = rh.rh_static_scratch_bytes()
    assert cap == 8 << 20
    t = torch.zeros(8, dtype=torch.int64, device=DEV)
    P = ctypes.c_void_p(t.data_ptr())
    marker = torch.full((4,), 5, dtype=torch.int64, device=DEV)
    M = ctypes.c_void_p(marker.data_ptr())
    assert rh.rh_workspace_size(rh.WS_STAGE_DP_WINDOW, 1, 65536, 64) <= cap
    assert rh.rh_workspace_size(rh.WS_STAGE_DP_WINDOW, 8, 65536, 64) > cap
    assert lib.rh_stage_dp_window_static(8, 65536, 64, P, None, 1, 2, M, P, None, None) == -7      # nothing launched
    assert lib.rh_stage_dp_window_static(1, 64, 65, P, None, 1, 2, M, P, None, None) == -2
    assert lib.rh_stage_dp_window_static(1, 64, 8, None, None, 1, 2, M, P, None, None) == -1
    assert lib.rh_stage_dp_window_static(0, 64, 8, None, None, 1, 2, None, None, None, None) == 0
    torch.cuda.synchronize()
    assert marker.tolist() == [5, 5, 5, 5]
    assert "static" in rh.strerror(-7)
