"""The five named workloads at full size on the GPU, against the CPU oracle (bit-exact).

Where the oracle cannot redo everything in seconds it checks a seeded sample of
problems or edges in full, and properties that need no oracle cover the rest
(the returned plan's objective, recomputed by plain gathers, equals the
returned total for every problem).
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import device_fill, graphs, synthetic as syn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
INF = oracle.INF


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def gpu_reshard(g, n_edges=None):
    n_edges = g["N"] - 1 if n_edges is None else n_edges
    Kp = g["Kp"]
    R = torch.empty((n_edges, Kp, Kp), dtype=torch.int64, device=DEV)
    rh.rh_build_reshard(rh.Mesh.make(g["m"], g["bw_bytes_per_us"], g["alpha_ns"]), n_edges, Kp, dev(g["K"]),
                        dev(g["out_spec"].view(np.int32)), dev(g["in_spec"].view(np.int32)), dev(g["dims"]),
                        dev(g["elem_bytes"]), R)
    return R


def gpu_chain(c, R, B, N, Kp, r_stride=None, workspace=False):
    arg = torch.empty((B, N - 1, Kp), dtype=torch.int16, device=DEV)
    total = torch.empty(B, dtype=torch.int64, device=DEV)
    last = torch.empty(B, dtype=torch.int32, device=DEV)
    plan = torch.empty((B, N), dtype=torch.int32, device=DEV)
    ws = None
    if workspace:
        ws = torch.empty(rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, B, N, Kp), dtype=torch.uint8, device=DEV)
        assert ws.numel() > 0
    rh.rh_minplus_chain(B, N, Kp, c, N * Kp, R, (N - 1) * Kp * Kp if r_stride is None else r_stride, arg, None,
                        total, last, ws)
    rh.rh_backtrack(B, N, Kp, arg, last, plan)
    torch.cuda.synchronize()
    return arg, total, last, plan


def objective_of_plans(c, R, plan):
    """sum_i c_i[x_i] + sum_i R_i[x_i][x_{i+1}] per problem, by plain gathers (c[B][N][K], R[B][N-1][K][K])."""
    B, N, K = c.shape
    x = plan.long()
    node = torch.gather(c, 2, x.unsqueeze(2)).squeeze(2).sum(1)
    flat = R.reshape(B, N - 1, K * K)
    edge = torch.gather(flat, 2, (x[:, :-1] * K + x[:, 1:]).unsqueeze(2)).squeeze(2).sum(1)
    return node + edge


def test_gpt_like_chain_with_mesh_enumeration():
    g = graphs.gpt_chain()
    N, Kp = g["N"], g["Kp"]
    assert N == 242 and Kp == 64
    R = gpu_reshard(g)
    want_R = oracle.build_reshard(g["m"], g["bw_bytes_per_us"], g["alpha_ns"], g["K"], g["out_spec"], g["in_spec"],
                                  g["dims"], g["elem_bytes"])
    torch.cuda.synchronize()
    assert np.array_equal(R.cpu().numpy(), want_R)
    c = dev(g["c"][None])
    arg, total, last, plan = gpu_chain(c, R, 1, N, Kp)
    o_arg, _, o_total, o_last = oracle.chain(g["c"][None], want_R[None])
    assert total.item() == o_total[0] < INF and last.item() == o_last[0]
    assert np.array_equal(arg.cpu().numpy().view(np.uint16), o_arg)
    assert np.array_equal(plan.cpu().numpy(), oracle.backtrack(o_arg, o_last))

    # the seven power-of-two shapes of a 64-device mesh as one batch (mesh shapes are searched in parallel)
    shapes = [(1 << k, 64 >> k) for k in range(7)]
    Rs, cs = [], []
    for m in shapes:
        gm = graphs.gpt_chain(m=m)
        Rs.append(gpu_reshard(gm))
        cs.append(gm["c"])
        o_R = oracle.build_reshard(m, g["bw_bytes_per_us"], g["alpha_ns"], gm["K"], gm["out_spec"], gm["in_spec"],
                                   gm["dims"], gm["elem_bytes"])
        torch.cuda.synchronize()
        assert np.array_equal(Rs[-1].cpu().numpy(), o_R), m
    Rb, cb = torch.stack(Rs).contiguous(), np.stack(cs)
    arg, total, last, plan = gpu_chain(dev(cb), Rb, 7, N, Kp)
    o_arg, _, o_total, o_last = oracle.chain(cb, Rb.cpu().numpy(), nthreads=4)
    assert np.array_equal(total.cpu().numpy(), o_total) and np.array_equal(last.cpu().numpy(), o_last)
    assert np.array_equal(plan.cpu().numpy(), oracle.backtrack(o_arg, o_last))
    assert o_total.min() < INF


def test_batched_random_chains_full_size():
    w = syn.BATCHED_CHAINS
    B, N, K = w["B"], w["N"], w["K"]
    need = B * ((N - 1) * K * K * 8 + N * K * 8 + (N - 1) * K * 2 + N * 4)
    free, _ = torch.cuda.mem_get_info()
    if free < need + (4 << 30):
        pytest.skip(f"needs {need / 2**30:.0f} GiB of free HBM, {free / 2**30:.0f} GiB available")
    c = torch.empty((B, N, K), dtype=torch.int64, device=DEV)
    R = torch.empty((B, N - 1, K, K), dtype=torch.int64, device=DEV)
    for p0 in range(0, B, 256):
        device_fill.fill_random_chain(c[p0:p0 + 256], R[p0:p0 + 256], p0, w["c_range"], w["r_range"])
    arg, total, last, plan = gpu_chain(c, R, B, N, K)       # the launch bench.py times
    # every problem: the plan's objective, recomputed by gathers, is the reported total
    obj = objective_of_plans(c, R, plan)
    assert torch.equal(obj, total)
    assert int(plan.min()) >= 0 and int(plan.max()) < K and torch.equal(plan[:, -1], last)
    # the device-side generator is the seeded twin of the host generator: a sample of its problems is regenerated
    # on the host and compared element by element
    sample = [0, 1, 255, 256, 1777, 2048, 3333, B - 1]
    hc, hR = syn.random_chain_batch(sample, N, K, w["c_range"], w["r_range"])
    idx = torch.tensor(sample, device=DEV)
    assert np.array_equal(c[idx].cpu().numpy(), hc) and np.array_equal(R[idx].cpu().numpy(), hR)
    del hc, hR
    # 264 seeded problems in full against the oracle (every arg row, total, last, plan): the eight above, plus 256
    # spread over the batch by a fixed stride that is coprime to the wave, workgroup and fill-slice sizes
    picked = sorted(set(sample) | {(7 + 13 * t) % B for t in range(256)})
    assert len(picked) >= 256
    for s0 in range(0, len(picked), 32):
        part = picked[s0:s0 + 32]
        pidx = torch.tensor(part, device=DEV)
        hc, hR = c[pidx].cpu().numpy(), R[pidx].cpu().numpy()
        o_arg, _, o_total, o_last = oracle.chain(hc, hR, nthreads=8)
        assert np.array_equal(total[pidx].cpu().numpy(), o_total), part
        assert np.array_equal(last[pidx].cpu().numpy(), o_last), part
        assert np.array_equal(arg[pidx].cpu().numpy().view(np.uint16), o_arg), part
        assert np.array_equal(plan[pidx].cpu().numpy(), oracle.backtrack(o_arg, o_last)), part
    # total and last of a further 1024 problems (every fourth), the oracle run on them in slices
    for s0 in range(2, B, 4 * 64):
        part = list(range(s0, min(B, s0 + 4 * 64), 4))
        pidx = torch.tensor(part, device=DEV)
        _, _, o_total, o_last = oracle.chain(c[pidx].cpu().numpy(), R[pidx].cpu().numpy(), nthreads=8)
        assert np.array_equal(total[pidx].cpu().numpy(), o_total), s0
        assert np.array_equal(last[pidx].cpu().numpy(), o_last), s0


def test_moe_shaped_graph_full_size():
    g = graphs.moe_chain()
    N, Kp = g["N"], g["Kp"]
    assert N == 8192 and Kp == 256
    R = gpu_reshard(g)                                       # 8191 x 256 x 256 tables, 4.29 GB, built on the device
    # the oracle counts units for one period of the layer pattern, the seam to the next layer and the tail;
    # the host arrays are periodic, so every other edge repeats one of those
    per, layers = 85, 96
    body = per * layers
    for name in ("out_spec", "in_spec", "c"):
        a = g[name][:body].reshape(layers, per, Kp)
        assert np.array_equal(a, np.broadcast_to(a[0], a.shape))
    dm = g["dims"][:body - 1]
    assert all(np.array_equal(dm[e], dm[e % per]) for e in range(0, body - 1, 7))
    first = oracle.build_reshard(g["m"], g["bw_bytes_per_us"], g["alpha_ns"], g["K"][:per + 1], g["out_spec"][:per + 1],
                                 g["in_spec"][:per + 1], g["dims"][:per], g["elem_bytes"][:per])
    t0 = body - 1                                            # edges from the last layer into and through the tail
    tail = oracle.build_reshard(g["m"], g["bw_bytes_per_us"], g["alpha_ns"], g["K"][t0:], g["out_spec"][t0:],
                                g["in_spec"][t0:], g["dims"][t0:], g["elem_bytes"][t0:])
    want = np.empty((N - 1, Kp, Kp), dtype=np.int64)
    for e in range(t0):
        want[e] = first[e % per]
    want[t0:] = tail
    torch.cuda.synchronize()
    got = R.cpu().numpy()
    assert np.array_equal(got, want)
    c = dev(g["c"][None])
    o_arg, _, o_total, o_last = oracle.chain(g["c"][None], want[None])
    o_plan = oracle.backtrack(o_arg, o_last)
    for workspace in (False, True):                          # one workgroup, then cut into segments
        arg, total, last, plan = gpu_chain(c, R, 1, N, Kp, workspace=workspace)
        assert total.item() == o_total[0] < INF and last.item() == o_last[0]
        assert np.array_equal(arg.cpu().numpy().view(np.uint16), o_arg)
        assert np.array_equal(plan.cpu().numpy(), o_plan)
    # and without any table in memory: every entry computed from the spec words, the chain cut into segments
    del R
    arg = torch.full((1, N - 1, Kp), -1, dtype=torch.int16, device=DEV)
    total = torch.zeros(1, dtype=torch.int64, device=DEV)
    last = torch.full((1,), -1, dtype=torch.int32, device=DEV)
    plan = torch.full((1, N), -1, dtype=torch.int32, device=DEV)
    ws = torch.full((rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SPECS, 1, N, Kp),), 0x11, dtype=torch.uint8, device=DEV)
    assert ws.numel() > 0
    rh.rh_minplus_chain_specs(1, N, Kp, [rh.Mesh.make(g["m"], g["bw_bytes_per_us"], g["alpha_ns"])], c, N * Kp,
                              dev(g["K"]), dev(g["out_spec"].view(np.int32)), dev(g["in_spec"].view(np.int32)),
                              dev(g["dims"]), dev(g["elem_bytes"]), arg, None, total, last, ws)
    rh.rh_backtrack(1, N, Kp, arg, last, plan)
    torch.cuda.synchronize()
    assert total.item() == o_total[0] and last.item() == o_last[0]
    assert np.array_equal(arg.cpu().numpy().view(np.uint16), o_arg)
    assert np.array_equal(plan.cpu().numpy(), o_plan)


def test_stage_partition_with_per_segment_chains():
    w = syn.STAGE_PARTITION
    L, S, M, K = w["L"], w["S"], w["seg_ops"], w["seg_K"]
    # every segment's cost is the total of its own chain of M operators with K candidates
    hc, hR = syn.random_chain_batch(range(L), M, K, w["seg_c_range"], w["seg_r_range"], c_lo=w["seg_c_lo"])
    c, R = dev(hc), dev(hR)
    dc = torch.empty_like(c)
    dR = torch.empty_like(R)
    device_fill.fill_random_chain(dc, dR, 0, w["seg_c_range"], w["seg_r_range"], c_lo=w["seg_c_lo"])
    assert torch.equal(dc, c) and torch.equal(dR, R)
    _, seg_cost, _, _ = gpu_chain(c, R, L, M, K)
    o_arg, _, o_total, o_last = oracle.chain(hc, hR, nthreads=8)
    assert np.array_equal(seg_cost.cpu().numpy(), o_total)
    bott = torch.empty((1, S), dtype=torch.int64, device=DEV)
    cut = torch.empty((1, S, L + 1), dtype=torch.int32, device=DEV)
    bounds = torch.empty((1, S + 1), dtype=torch.int32, device=DEV)
    ws = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP, 1, L, S), dtype=torch.uint8, device=DEV)
    rh.rh_stage_dp(1, L, S, seg_cost.reshape(1, L), bott, cut, S, bounds, ws)
    torch.cuda.synchronize()
    o_bott, o_cut, o_bounds = oracle.stage_dp(o_total[None], S, s_query=S, nthreads=1)
    assert np.array_equal(bott.cpu().numpy(), o_bott)
    assert np.array_equal(cut.cpu().numpy(), o_cut)
    assert np.array_equal(bounds.cpu().numpy(), o_bounds)
