"""The entry points only enqueue kernels on the caller's stream: they can be captured into a HIP graph and
replayed, and calls on different streams can overlap.  Every replay is checked against the eager result."""
import numpy as np
import pytest
import torch

import oracle
from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import synthetic as syn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def chain_buffers(B, N, Kp):
    return dict(arg=torch.zeros((B, N - 1, Kp), dtype=torch.int16, device=DEV),
                total=torch.zeros(B, dtype=torch.int64, device=DEV),
                last=torch.zeros(B, dtype=torch.int32, device=DEV),
                plan=torch.zeros((B, N), dtype=torch.int32, device=DEV))


def run_chain(c, R, o, ws=None):
    B, N, Kp = c.shape
    rh.rh_minplus_chain(B, N, Kp, c, N * Kp, R, (N - 1) * Kp * Kp, o["arg"], None, o["total"], o["last"], ws)
    rh.rh_backtrack(B, N, Kp, o["arg"], o["last"], o["plan"])


@pytest.mark.parametrize("B,N,Kp,with_ws", [(9, 30, 128, False), (2, 80, 256, True), (2100, 3, 64, False),
                                            (1, 700, 64, True), (2, 300, 128, True)])   # the last two: long chains cut into segments
def test_graph_capture_and_replay(B, N, Kp, with_ws):
    hc, hR = syn.random_chain_batch(range(B), N, Kp, 1000, 5000)
    c, R = torch.from_numpy(hc).to(DEV), torch.from_numpy(hR).to(DEV)
    ws = None
    if with_ws:
        ws = torch.empty(rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, B, N, Kp), dtype=torch.uint8, device=DEV)
        assert ws.numel() > 0
    o = chain_buffers(B, N, Kp)
    L, S = 300, 12
    cost = torch.from_numpy(np.stack([syn.segment_costs(p, L) for p in range(2)])).to(DEV)
    bott = torch.zeros((2, S), dtype=torch.int64, device=DEV)
    cut = torch.zeros((2, S, L + 1), dtype=torch.int32, device=DEV)
    bounds = torch.zeros((2, S + 1), dtype=torch.int32, device=DEV)
    sws = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP, 2, L, S), dtype=torch.uint8, device=DEV)

    def work():
        run_chain(c, R, o, ws)
        rh.rh_stage_dp(2, L, S, cost, bott, cut, S, bounds, sws)

    work()                                                   # eager reference (and warm-up before capture)
    torch.cuda.synchronize()
    want = {k: v.clone() for k, v in o.items()}
    want_b, want_bounds = bott.clone(), bounds.clone()
    o_arg, _, o_total, o_last = oracle.chain(hc, hR, nthreads=8)
    assert np.array_equal(want["total"].cpu().numpy(), o_total)
    assert np.array_equal(want["plan"].cpu().numpy(), oracle.backtrack(o_arg, o_last))

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            work()
    torch.cuda.synchronize()
    for rep in range(3):
        for v in o.values():
            v.fill_(-1)                                      # eager work between the replays
        bott.fill_(-1)
        bounds.fill_(-1)
        if ws is not None:
            ws.fill_(rep + 1)                                # stale workspace contents must not matter
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        for k in o:
            assert torch.equal(o[k], want[k]), (rep, k)
        assert torch.equal(bott, want_b) and torch.equal(bounds, want_bounds), rep


def test_graph_of_the_stage_searches():
    # interval table + search over it, the windowed search, and the full-scan search of a chain beyond the LDS limit
    L, K, S = 150, 32, 9
    hc, hR = syn.random_chain_batch([3], L, K, 1000, 5000)
    c, R = torch.from_numpy(hc).to(DEV), torch.from_numpy(hR).to(DEV)
    ldT = L + 2 - (L & 1)
    T = torch.zeros((1, L, ldT), dtype=torch.int64, device=DEV)
    out = {"b1": torch.zeros((1, S), dtype=torch.int64, device=DEV),
           "c1": torch.zeros((1, S, L + 1), dtype=torch.int32, device=DEV),
           "d1": torch.zeros((1, S + 1), dtype=torch.int32, device=DEV),
           "b2": torch.zeros(1, dtype=torch.int64, device=DEV),
           "c2": torch.zeros((1, S, L + 1), dtype=torch.int32, device=DEV),
           "d2": torch.zeros((1, S + 1), dtype=torch.int32, device=DEV)}
    Lb = 6200
    cost = torch.from_numpy(syn.segment_costs(1, L)[None]).to(DEV)
    costb = torch.from_numpy(syn.segment_costs(2, Lb)[None]).to(DEV)
    out["b3"] = torch.zeros((1, 4), dtype=torch.int64, device=DEV)
    out["c3"] = torch.zeros((1, 4, Lb + 1), dtype=torch.int32, device=DEV)
    w1 = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP_INTERVAL, 1, L, S), dtype=torch.uint8, device=DEV)
    w2 = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP_WINDOW, 1, L, S), dtype=torch.uint8, device=DEV)
    w3 = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP, 1, Lb, 4), dtype=torch.uint8, device=DEV)

    def work():
        rh.rh_interval_costs(1, L, K, c, R, ldT, T)
        rh.rh_stage_dp_interval(1, L, S, ldT, T, out["b1"], out["c1"], S, out["d1"], w1)
        rh.rh_stage_dp_window(1, L, S, cost, None, 1, 1, out["b2"], out["c2"], out["d2"], w2)
        rh.rh_stage_dp(1, Lb, 4, costb, out["b3"], out["c3"], 0, None, w3)

    work()
    torch.cuda.synchronize()
    want = {k: v.clone() for k, v in out.items()}
    want_T = T.clone()
    o_T = oracle.interval_costs(hc[0], hR[0], ldT=ldT)
    assert np.array_equal(want_T.cpu().numpy()[0, :, :L + 1], o_T[:, :L + 1])
    o_b, o_c, o_d = oracle.stage_interval(o_T[None], S, s_query=S)
    assert np.array_equal(want["b1"].cpu().numpy(), o_b) and np.array_equal(want["d1"].cpu().numpy(), o_d)
    assert np.array_equal(want["b3"].cpu().numpy(), oracle.stage_dp(costb.cpu().numpy(), 4)[0])

    g = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(g, stream=side):
            work()
    torch.cuda.synchronize()
    for rep in range(3):
        for v in out.values():
            v.fill_(-1)
        T.fill_(-1)
        for w in (w1, w2, w3):
            w.fill_(rep + 1)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(T[0, :, :L + 1], want_T[0, :, :L + 1]), rep
        for k in out:
            assert torch.equal(out[k], want[k]), (rep, k)


def test_calls_on_two_streams_overlap_safely():
    B, N, Kp = 64, 60, 128
    data = []
    for base in (0, 1000):
        hc, hR = syn.random_chain_batch(range(base, base + B), N, Kp, 1000, 5000)
        data.append((hc, hR, torch.from_numpy(hc).to(DEV), torch.from_numpy(hR).to(DEV), chain_buffers(B, N, Kp)))
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for _ in range(3):
        for s, (_, _, c, R, o) in zip(streams, data):
            with torch.cuda.stream(s):
                run_chain(c, R, o)
    torch.cuda.synchronize()
    for hc, hR, _, _, o in data:
        o_arg, _, o_total, o_last = oracle.chain(hc, hR, nthreads=8)
        assert np.array_equal(o["total"].cpu().numpy(), o_total)
        assert np.array_equal(o["plan"].cpu().numpy(), oracle.backtrack(o_arg, o_last))
