"""GPU parity of the chain DP that computes resharding times on the fly (rh_minplus_chain_specs) against the
oracle's unit-counting tables + chain DP (bit-exact), one logical mesh per problem."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import graphs, specs as sp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
INF = oracle.INF


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def gpu_fused(g, meshes, cs, segmented=False):
    """g: graph dict (specs shared); meshes: list of (m, bw, alpha); cs: [B][N][Kp] node costs; segmented: with the
    workspace that cuts the chains into segments (stale contents)."""
    B, N, Kp = cs.shape
    ws = None
    if segmented:
        need = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SPECS, B, N, Kp)
        assert need > 0
        ws = torch.full((need,), 0x6D, dtype=torch.uint8, device=DEV)
    arg = torch.full((B, N - 1, Kp), -1, dtype=torch.int16, device=DEV)
    vfinal = torch.zeros((B, Kp), dtype=torch.int64, device=DEV)
    total = torch.zeros(B, dtype=torch.int64, device=DEV)
    last = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    plan = torch.full((B, N), -1, dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain_specs(B, N, Kp, [rh.Mesh.make(*m) for m in meshes], dev(cs), N * Kp, dev(g["K"]),
                              dev(g["out_spec"].view(np.int32)), dev(g["in_spec"].view(np.int32)), dev(g["dims"]),
                              dev(g["elem_bytes"]), arg, vfinal, total, last, ws)
    rh.rh_backtrack(B, N, Kp, arg, last, plan)
    torch.cuda.synchronize()
    return arg.cpu().numpy().view(np.uint16), vfinal.cpu().numpy(), total.cpu().numpy(), last.cpu().numpy(), \
        plan.cpu().numpy()


def check(g, meshes, cs, segmented=(False,)):
    want = []
    for p, (m, bw, alpha) in enumerate(meshes):
        R = oracle.build_reshard(m, bw, alpha, g["K"], g["out_spec"], g["in_spec"], g["dims"], g["elem_bytes"])
        o_arg, o_vf, o_total, o_last = oracle.chain(np.ascontiguousarray(cs[p][None]), R[None])
        want.append((o_arg[0], o_vf[0], o_total[0], o_last[0], oracle.backtrack(o_arg, o_last)[0]))
    for seg in segmented:
        got = gpu_fused(g, meshes, cs, seg)
        for p, (m, bw, alpha) in enumerate(meshes):
            assert got[2][p] == want[p][2] and got[3][p] == want[p][3], (p, m, seg)
            assert np.array_equal(got[1][p], want[p][1]), (p, m, seg)
            assert np.array_equal(got[0][p], want[p][0]), (p, m, seg)
            assert np.array_equal(got[4][p], want[p][4]), (p, m, seg)
    return got[2]


def test_gpt_like_chain_over_the_mesh_shapes_of_64_devices():
    shapes = [(1 << k, 64 >> k) for k in range(7)]
    gs = [graphs.gpt_chain(m=m) for m in shapes]
    meshes = [(m, g["bw_bytes_per_us"], (0, 250)) for m, g in zip(shapes, gs)]
    totals = check(gs[0], meshes, np.stack([g["c"] for g in gs]), segmented=(False, True))
    assert totals.min() < INF


@pytest.mark.parametrize("Kp", [64, 128, 256])
def test_random_spec_words_and_ragged_candidates(Kp):
    rng = np.random.default_rng(Kp)
    N = 9
    out_spec = rng.integers(0, 1 << 16, size=(N, Kp)).astype(np.uint32)
    in_spec = rng.integers(0, 1 << 16, size=(N, Kp)).astype(np.uint32)
    # make a good share of the words valid layouts: states 0..2, dims 0..3, small lgdiv
    ok = rng.random((N, Kp)) < 0.7
    def tidy(w):
        b0 = (w & 3) % 3 | (((w >> 2) & 3) << 2) | (((w >> 5) & 1) << 5)
        b1 = ((w >> 8) & 3) % 3 | ((((w >> 10) & 3)) << 2) | ((((w >> 13) & 1)) << 5)
        return (b0 | (b1 << 8)).astype(np.uint32)
    out_spec = np.where(ok, tidy(out_spec), out_spec)
    in_spec = np.where(ok, tidy(in_spec), in_spec)
    out_spec[:, ::11] = sp.EMPTY
    g = dict(K=rng.integers(Kp // 2, Kp + 1, size=N).astype(np.int32), out_spec=out_spec, in_spec=in_spec,
             dims=np.tile(np.array([[64, 128, 256, 512]], dtype=np.int64), (N - 1, 1)),
             elem_bytes=np.full(N - 1, 2, dtype=np.int32))
    meshes = [((4, 8), (12500, 150000), (5, 0)), ((32,), (50000,), (0,)), ((2, 2), (1000, 1000), (0, 0))]
    cs = rng.integers(0, 100000, size=(3, N, Kp)).astype(np.int64)
    cs[rng.random(cs.shape) < 0.1] = INF
    check(g, meshes, cs)


def test_more_problems_than_meshes():
    g = graphs.gpt_chain(layers=2)
    meshes = [((8, 8), g["bw_bytes_per_us"], (0, 0)), ((4, 16), g["bw_bytes_per_us"], (0, 0)),
              ((64, 1), g["bw_bytes_per_us"], (7, 7))]
    rng = np.random.default_rng(1)
    B = 8
    cs = np.stack([np.where(g["c"] < INF, g["c"] + rng.integers(0, 1000), INF) for _ in range(B)])
    got = gpu_fused(g, meshes, cs)
    for p in range(B):
        m, bw, alpha = meshes[p % 3]
        R = oracle.build_reshard(m, bw, alpha, g["K"], g["out_spec"], g["in_spec"], g["dims"], g["elem_bytes"])
        o_arg, _, o_total, o_last = oracle.chain(np.ascontiguousarray(cs[p][None]), R[None])
        assert got[2][p] == o_total[0] and np.array_equal(got[0][p], o_arg[0])


def test_moe_shaped_graph_prefix():
    g = graphs.moe_chain(layers=2, tail=3)                   # 173 operators, K = 256, two mesh shapes
    g2 = graphs.moe_chain(layers=2, tail=3)
    meshes = [((32, 32), g["bw_bytes_per_us"], (0, 0)), ((16, 64), g["bw_bytes_per_us"], (100, 0))]
    cs = np.stack([g["c"], g2["c"] // 2])
    check(g, meshes, cs)


@pytest.mark.parametrize("Kp,N", [(64, 128), (64, 500), (128, 333), (256, 260), (256, 700)])
def test_segmented_route_on_random_spec_words(Kp, N):
    # long chains cut into segments, every table entry computed from the words: random words (valid layouts,
    # invalid ones, empty slots), ragged candidate counts, infeasible node costs, three meshes (one with one axis)
    rng = np.random.default_rng(Kp * 1000 + N)
    words = rng.integers(0, 1 << 16, size=(2, N, Kp)).astype(np.uint32)
    ok = rng.random((2, N, Kp)) < 0.8
    b0 = (words & 3) % 3 | (((words >> 2) & 3) << 2) | (((words >> 5) & 1) << 5)
    b1 = ((words >> 8) & 3) % 3 | (((words >> 10) & 3) << 2) | (((words >> 13) & 1) << 5)
    words = np.where(ok, (b0 | (b1 << 8)).astype(np.uint32), words)
    words[0, :, ::13] = sp.EMPTY
    dims = np.tile(np.array([[64, 128, 256, 512]], dtype=np.int64), (N - 1, 1))
    dims[::5] = [96, 64, 48, 1]                               # extents that some strides do not divide
    g = dict(K=rng.integers(Kp // 2, Kp + 1, size=N).astype(np.int32), out_spec=words[0], in_spec=words[1],
             dims=dims, elem_bytes=rng.choice([1, 2, 4], size=N - 1).astype(np.int32))
    meshes = [((4, 8), (12500, 150000), (5, 0)), ((32,), (50000,), (0,)), ((2, 2), (1000, 1000), (0, 3))]
    cs = rng.integers(0, 100000, size=(3, N, Kp)).astype(np.int64)
    cs[rng.random(cs.shape) < 0.3] = INF
    cs[:, :, 1] = 7                                           # one strategy stays in the game at every operator...
    g["out_spec"][:, 1] = sp.word(sp.R_, sp.R_)                # ...and its layouts are valid
    g["in_spec"][:, 1] = sp.word(sp.R_, sp.R_)
    cs[2, N // 2:, :] = np.where(rng.random((N - N // 2, Kp)) < 0.9, INF, cs[2, N // 2:, :])   # a sparse second half
    cs[2, :, 1] = 7
    totals = check(g, meshes, cs, segmented=(True,))
    assert (totals < INF).all()


def test_segmented_route_when_the_chain_dies():
    g = graphs.gpt_chain(layers=20)
    N, Kp = g["N"], g["Kp"]
    cs = np.stack([g["c"], g["c"]])
    cs[1, 150, :] = INF                                       # nothing is feasible from operator 150 on
    meshes = [((8, 8), g["bw_bytes_per_us"], (0, 0))]
    got = gpu_fused(g, meshes, cs, segmented=True)
    R = oracle.build_reshard((8, 8), g["bw_bytes_per_us"], (0, 0), g["K"], g["out_spec"], g["in_spec"], g["dims"],
                             g["elem_bytes"])
    o_arg, o_vf, o_total, o_last = oracle.chain(cs, R, shared_R=True)
    assert o_total[1] == INF and o_total[0] < INF
    assert np.array_equal(got[2], o_total) and np.array_equal(got[3], o_last)
    assert np.array_equal(got[1], o_vf) and np.array_equal(got[0], o_arg)


def test_argument_errors():
    L = rh.lib()
    t = torch.zeros(64 * 64 * 2, dtype=torch.int64, device=DEV)
    P = ctypes.c_void_p(t.data_ptr())
    good = (rh.Mesh * 1)(rh.Mesh.make((8, 8), (1000, 1000)))
    bad = (rh.Mesh * 1)(rh.Mesh.make((6, 8), (1000, 1000)))
    call = lambda B=1, N=2, Kp=64, m=good, nm=1: L.rh_minplus_chain_specs(B, N, Kp, nm, m, P, 128, P, P, P, P, P, P,
                                                                          None, P, P, None, 0, None)
    assert call(Kp=32) == -3 and call(Kp=512) == -3 and call(nm=65) == -2 and call(nm=0) == -2 and call(N=0) == -2
    assert call(m=bad) == -2 and call(m=None) == -1 and call(B=0) == 0
    # a workspace is 256-byte aligned; a short one is simply not used
    assert L.rh_minplus_chain_specs(1, 2, 64, 1, good, P, 128, P, P, P, P, P, P, None, P, P,
                                    ctypes.c_void_p(t.data_ptr() + 8), 64, None) == -4
    assert rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SPECS, 1, 127, 64) == 0
    assert rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SPECS, 33, 500, 64) == 0
    assert rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SPECS, 1, 500, 512) == 0
    torch.cuda.synchronize()


def test_single_operator_needs_no_specs():
    # one operator, no edge: v_0 = c_0, and none of the spec arrays is looked at (they may be missing)
    rng = np.random.default_rng(5)
    B, Kp = 3, 64
    c = rng.integers(0, 1000, size=(B, 1, Kp)).astype(np.int64)
    c[1, 0, :] = INF
    c[2, 0, :7] = INF
    vfinal = torch.zeros((B, Kp), dtype=torch.int64, device=DEV)
    total = torch.zeros(B, dtype=torch.int64, device=DEV)
    last = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain_specs(B, 1, Kp, [rh.Mesh.make((8, 8), (12_500, 150_000), (0, 0))], dev(c), Kp, None, None, None,
                              None, None, None, vfinal, total, last)
    torch.cuda.synchronize()
    _, o_vf, o_total, o_last = oracle.chain(c, np.zeros((B, 0, Kp, Kp), dtype=np.int64))
    assert np.array_equal(total.cpu().numpy(), o_total) and np.array_equal(last.cpu().numpy(), o_last)
    assert np.array_equal(vfinal.cpu().numpy(), o_vf)
