"""The cost contract at its ceiling on every route of the chain DP (bit-exact against the CPU oracle).

The interface allows finite costs below 2^36 and chains of up to 2^14 operators, so totals approach 2^51.  The
routes differ in their arithmetic (64-bit integer keys, packed (cost, index) words, fp64 min-plus inside the
segmented route), so each of them is run at that ceiling: the longest chain, every finite cost within 2^10 of 2^36,
some strategies and pairs infeasible.
"""
import numpy as np
import pytest
import torch

import oracle
from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import specs as sp

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
INF = oracle.INF
N_MAX = 16384
TOP = 1 << 36


def ceiling_tables(B, Kp, seed):
    rng = np.random.default_rng(seed)
    c = rng.integers(TOP - 1024, TOP, size=(B, N_MAX, Kp), dtype=np.int64)
    R = rng.integers(TOP - 1024, TOP, size=(B, N_MAX - 1, Kp, Kp), dtype=np.int64)
    for p in range(B):
        # whole strategies infeasible (row of the table that leaves the operator, column of the one that arrives)
        for i in rng.choice(N_MAX, size=N_MAX // 16, replace=False):
            dead = rng.choice(np.arange(1, Kp), size=int(rng.integers(1, Kp // 2)), replace=False)
            c[p, i, dead] = INF
            if i < N_MAX - 1:
                R[p, i, dead, :] = INF
            if i > 0:
                R[p, i - 1, :, dead] = INF
        # and single pairs that cannot be converted
        for i in rng.choice(N_MAX - 1, size=N_MAX // 16, replace=False):
            R[p, i][rng.random((Kp, Kp)) < 0.05] = INF
    return c, R


def run_route(dc, dR, B, Kp, ws):
    arg = torch.full((B, N_MAX - 1, Kp), -1, dtype=torch.int16, device=DEV)
    vfinal = torch.zeros((B, Kp), dtype=torch.int64, device=DEV)
    total = torch.zeros(B, dtype=torch.int64, device=DEV)
    last = torch.full((B,), -1, dtype=torch.int32, device=DEV)
    plan = torch.full((B, N_MAX), -1, dtype=torch.int32, device=DEV)
    rh.rh_minplus_chain(B, N_MAX, Kp, dc, N_MAX * Kp, dR, (N_MAX - 1) * Kp * Kp, arg, vfinal, total, last, ws)
    rh.rh_backtrack(B, N_MAX, Kp, arg, last, plan)
    torch.cuda.synchronize()
    return arg.cpu().numpy().view(np.uint16), vfinal.cpu().numpy(), total.cpu().numpy(), last.cpu().numpy(), \
        plan.cpu().numpy()


@pytest.mark.parametrize("Kp", [64, 128])
def test_table_routes_at_the_cost_ceiling(Kp):
    B = 3
    c, R = ceiling_tables(B, Kp, seed=Kp)
    o_arg, o_vf, o_total, o_last = oracle.chain(c, R, nthreads=8)
    o_plan = oracle.backtrack(o_arg, o_last)
    assert (o_total < INF).all() and o_total.min() > (N_MAX * 2 - 1) * (TOP - 1024)   # about 2^51
    dc, dR = torch.from_numpy(c).to(DEV), torch.from_numpy(R).to(DEV)

    def same(got, sel, route):
        for g, o in zip(got, (o_arg, o_vf, o_total, o_last, o_plan)):
            assert np.array_equal(g, o[sel]), route

    routes = [("one workgroup per problem", B, None)]
    gang = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, B, N_MAX, Kp)
    if Kp >= 128:
        assert gang > 0
        routes.append(("eight workgroups per problem", B, gang))
    else:
        assert gang == 0
    one = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, 1, N_MAX, Kp)
    seg = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SEGMENTED, B, N_MAX, Kp)
    assert one > 0 and seg > gang
    routes += [("segments, one problem", 1, one), ("segments, three problems", B, seg)]
    for route, nb, nbytes in routes:
        ws = None if nbytes is None else torch.full((nbytes,), 0xC3, dtype=torch.uint8, device=DEV)
        same(run_route(dc[:nb], dR[:nb], nb, Kp, ws), slice(0, nb), route)


def test_spec_route_at_the_cost_ceiling():
    # node costs within 2^10 of 2^36; resharding times from the spec words of a 4x4 mesh, the dearest (all-gather of
    # the whole 2^26-byte tensor at 2 bytes per microsecond, after the other axis was gathered) 2.8e10 ns
    Kp, period = 64, 16
    rng = np.random.default_rng(36)
    opts = [sp.R_] + [sp.S_(d, lg) for d in range(3) for lg in (0, 1)]
    words = np.array([sp.word(a, b) for a in opts for b in opts], dtype=np.uint32)      # 49, some split one dim twice
    out_p = np.full((period, Kp), sp.EMPTY, dtype=np.uint32)
    in_p = np.full((period, Kp), sp.EMPTY, dtype=np.uint32)
    K_p = rng.integers(40, Kp + 1, size=period).astype(np.int32)
    for i in range(period):
        out_p[i, :K_p[i]] = rng.choice(words, size=K_p[i])
        in_p[i, :K_p[i]] = rng.choice(words, size=K_p[i])
    reps = N_MAX // period
    g = dict(K=np.tile(K_p, reps), out_spec=np.tile(out_p, (reps, 1)), in_spec=np.tile(in_p, (reps, 1)),
             dims=np.tile(np.array([[256, 256, 512, 1]], dtype=np.int64), (N_MAX - 1, 1)),
             elem_bytes=np.full(N_MAX - 1, 2, dtype=np.int32))
    mesh = ((4, 4), (2, 2), (0, 3))
    # the oracle counts units for one period and the seam back to its start; every other edge repeats one of those
    idx = list(range(period)) + [0]
    R_p = oracle.build_reshard(mesh[0], mesh[1], mesh[2], g["K"][idx], g["out_spec"][idx], g["in_spec"][idx],
                               g["dims"][:period], g["elem_bytes"][:period])
    finite = R_p[R_p < INF]
    assert finite.max() < TOP and finite.max() > (1 << 34)
    R = np.ascontiguousarray(np.tile(R_p, (reps, 1, 1))[:N_MAX - 1])
    c = rng.integers(TOP - 1024, TOP, size=(1, N_MAX, Kp), dtype=np.int64)
    c[0][np.arange(Kp)[None, :] >= g["K"][:, None]] = INF
    o_arg, o_vf, o_total, o_last = oracle.chain(c, R[None])
    assert N_MAX * (TOP - 1024) <= o_total[0] < INF         # 2^50 and more

    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    need = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SPECS, 1, N_MAX, Kp)
    assert need > 0
    for ws in (None, torch.full((need,), 0x2E, dtype=torch.uint8, device=DEV)):   # edge by edge, then in segments
        arg = torch.full((1, N_MAX - 1, Kp), -1, dtype=torch.int16, device=DEV)
        vfinal = torch.zeros((1, Kp), dtype=torch.int64, device=DEV)
        total = torch.zeros(1, dtype=torch.int64, device=DEV)
        last = torch.full((1,), -1, dtype=torch.int32, device=DEV)
        rh.rh_minplus_chain_specs(1, N_MAX, Kp, [rh.Mesh.make(*mesh)], d(c), N_MAX * Kp, d(g["K"]),
                                  d(g["out_spec"].view(np.int32)), d(g["in_spec"].view(np.int32)), d(g["dims"]),
                                  d(g["elem_bytes"]), arg, vfinal, total, last, ws)
        torch.cuda.synchronize()
        assert total.item() == o_total[0] and last.item() == o_last[0], ws is None
        assert np.array_equal(vfinal.cpu().numpy(), o_vf)
        assert np.array_equal(arg.cpu().numpy().view(np.uint16), o_arg)
