"""GPU parity of the memory-constrained search (Sec. 4.4) against the CPU oracle (bit-exact)."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import graphs

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
INF = oracle.INF


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def gpu_sweep(c, R, param_bytes, repl, mem, limit, n_k, k0=0, use_workspace=False):
    """One chain batch over k = k0 .. k0+n_k-1 with shared edge tables."""
    N, Kp = c.shape
    dR = R if isinstance(R, torch.Tensor) else dev(R)
    cm = torch.full((n_k, N, Kp), -7, dtype=torch.int64, device=DEV)
    rh.rh_mask_replicated(N, Kp, n_k, k0, dev(c), dev(param_bytes), dev(repl), cm)
    arg = torch.empty((n_k, N - 1, Kp), dtype=torch.int16, device=DEV)
    total = torch.empty(n_k, dtype=torch.int64, device=DEV)
    last = torch.empty(n_k, dtype=torch.int32, device=DEV)
    plan = torch.empty((n_k, N), dtype=torch.int32, device=DEV)
    ws = None
    if use_workspace:                             # True: the default kind; else the kind named
        kind = rh.WS_MINPLUS_CHAIN if use_workspace is True else use_workspace
        ws = torch.empty(rh.rh_workspace_size(kind, n_k, N, Kp), dtype=torch.uint8, device=DEV)
    rh.rh_minplus_chain(n_k, N, Kp, cm, N * Kp, dR, 0, arg, None, total, last, ws)
    rh.rh_backtrack(n_k, N, Kp, arg, last, plan)
    plan_mem = torch.full((n_k,), -7, dtype=torch.int64, device=DEV)
    first = torch.full((1,), -7, dtype=torch.int32, device=DEV)
    rh.rh_plan_memory(n_k, N, Kp, plan, dev(mem), total, limit, plan_mem, first)
    torch.cuda.synchronize()
    return total.cpu().numpy(), plan.cpu().numpy(), plan_mem.cpu().numpy(), int(first.item()), cm


def check(c, R_host, param_bytes, repl, mem, limit, n_k, k0=0, R_dev=None, use_workspace=False):
    o_total, o_plan, o_mem, o_first = oracle.memory_sweep(c, R_host, param_bytes, repl, mem, limit, n_k, k0)
    total, plan, plan_mem, first, _ = gpu_sweep(c, R_dev if R_dev is not None else R_host, param_bytes, repl, mem,
                                                limit, n_k, k0, use_workspace)
    assert np.array_equal(total, o_total)
    assert np.array_equal(plan, o_plan)
    assert np.array_equal(plan_mem, o_mem)
    assert first == o_first
    return o_total, o_first


@pytest.mark.parametrize("seed", range(4))
def test_random_chains(seed):
    rng = np.random.default_rng(seed)
    N, K, Kp = int(rng.integers(2, 40)), int(rng.integers(3, 60)), 64
    c = np.full((N, Kp), INF, dtype=np.int64)
    c[:, :K] = rng.integers(0, 1000, size=(N, K))
    R = np.full((N - 1, Kp, Kp), INF, dtype=np.int64)
    R[:, :K, :K] = rng.integers(0, 1000, size=(N - 1, K, K))
    pb = rng.integers(0, 5, size=N).astype(np.int64) * 4096                  # ties, operators without parameters
    repl = (rng.random((N, Kp)) < 0.5).astype(np.uint8)
    repl[:, 0] = 1
    if seed == 1:
        repl[N // 2] = 1                                                      # an operator that can only replicate
    mem = np.where(repl != 0, pb[:, None], pb[:, None] // 8).astype(np.int64)
    limit = int(mem.min(axis=1).sum() + rng.integers(0, 3 * 4096))
    check(c, R, pb, repl, mem, limit, N + 1)
    check(c, R, pb, repl, mem, limit, 3, k0=N // 2)
    check(c, R, pb, repl, mem, -1, 2)                                         # nothing fits: first = -1


def test_gpt_like_chain_sweep():
    g = graphs.gpt_chain()
    R = oracle.build_reshard(g["m"], g["bw_bytes_per_us"], g["alpha_ns"], g["K"], g["out_spec"], g["in_spec"],
                             g["dims"], g["elem_bytes"])
    n_params = int((g["param_bytes"] > 0).sum())
    assert n_params == 24 * 4 + 1
    replicated = int(g["param_bytes"].sum())
    least = int(g["mem"].min(axis=1).sum())
    # the unconstrained plan replicates every weight (pure data/sequence parallelism); a limit of an eighth forces
    # most of the largest ones to be split
    limit = replicated // 8
    assert least <= limit
    totals, first = check(g["c"], R, g["param_bytes"], g["repl"], g["mem"], limit, n_params + 1)
    assert 0 < first <= n_params and np.all(np.diff(totals) >= 0)


_moe = {}


def moe_tables():
    """The MoE-shaped graph with its tables from the oracle (host) and from rh_build_reshard (device), once."""
    if not _moe:
        g = graphs.moe_chain()
        N, Kp = g["N"], g["Kp"]
        R = torch.empty((N - 1, Kp, Kp), dtype=torch.int64, device=DEV)
        rh.rh_build_reshard(rh.Mesh.make(g["m"], g["bw_bytes_per_us"], g["alpha_ns"]), N - 1, Kp, dev(g["K"]),
                            dev(g["out_spec"].view(np.int32)), dev(g["in_spec"].view(np.int32)), dev(g["dims"]),
                            dev(g["elem_bytes"]), R)
        torch.cuda.synchronize()
        R_host = oracle.build_reshard(g["m"], g["bw_bytes_per_us"], g["alpha_ns"], g["K"], g["out_spec"], g["in_spec"],
                                      g["dims"], g["elem_bytes"])
        assert np.array_equal(R.cpu().numpy(), R_host)
        _moe.update(g=g, R=R, R_host=R_host)
    return _moe["g"], _moe["R"], _moe["R_host"]


def test_moe_shaped_graph_sweep_chunk():
    g, R, R_host = moe_tables()
    limit = 64 << 30
    # k = 190 .. 193 of the 480 parameters, once per kernel family (one workgroup per problem, then eight)
    for use_ws in (False, True):
        check(g["c"], R_host, g["param_bytes"], g["repl"], g["mem"], limit, 4, k0=190, R_dev=R, use_workspace=use_ws)


def test_moe_shaped_graph_sweep_of_the_timing_row():
    # 16 values of k from 176 under a limit of 2^40 bytes per device, all chains cut into segments (the workspace of
    # exactly the segmented size): the sweep ends at a feasible k
    g, R, R_host = moe_tables()
    totals, first = check(g["c"], R_host, g["param_bytes"], g["repl"], g["mem"], 1 << 40, 16, k0=176, R_dev=R,
                          use_workspace=rh.WS_MINPLUS_CHAIN_SEGMENTED)
    assert first == 10 and totals[first] < INF
    _moe.clear()


def test_argument_errors():
    L = rh.lib()
    t = torch.zeros(64 * 4, dtype=torch.int64, device=DEV)
    P = ctypes.c_void_p(t.data_ptr())
    assert L.rh_mask_replicated(4, 48, 1, 0, P, P, P, P, None) == -3
    assert L.rh_mask_replicated(0, 64, 1, 0, P, P, P, P, None) == -2
    assert L.rh_mask_replicated(4, 64, 1, 0, P, None, P, P, None) == -1
    assert L.rh_mask_replicated(4, 64, 0, 0, None, None, None, None, None) == 0
    assert L.rh_plan_memory(1, 4, 64, None, P, P, 0, P, None, None) == -1
    assert L.rh_plan_memory(-1, 4, 64, P, P, P, 0, P, None, None) == -2
    torch.cuda.synchronize()
