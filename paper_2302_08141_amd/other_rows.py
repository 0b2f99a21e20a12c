"""Timings of the path's other rows on their own workloads (called by bench.py after the timed steps).

Each figure is the best of a few repetitions, taken with events on the launch
stream, inputs resident on the device:
  * the MoE-shaped graph (8192 operators, K=256, logical 32x32 mesh): reshard tables from specs
    (4.29 GB written), chain DP and backtrack of the single long chain;
  * the GPT-like chain (242 operators, K=64, logical 8x8 mesh): the same three calls;
  * the stage partition (L=4096 segments, S=64): per-segment chains (8 operators, K=64) then the stage DP.
"""
from __future__ import annotations

import numpy as np
import torch

from . import binding as rh
from .workloads import cones as wc, device_fill, graphs, synthetic as syn


def _best_ms(fn, reps=3):
    best = None
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        fn()
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1)
        best = t if best is None or t < best else best
    return best


def _memory_sweep_rows(g, R, dev, n_k=16, k0=176):
    """Memory-constrained search on the graph: n_k values of k as one chain batch sharing the edge tables."""
    N, Kp = g["N"], g["Kp"]
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    c, pb, repl, mem = to(g["c"]), to(g["param_bytes"]), to(g["repl"]), to(g["mem"])
    cm = torch.empty((n_k, N, Kp), dtype=torch.int64, device=dev)
    arg = torch.empty((n_k, N - 1, Kp), dtype=torch.int16, device=dev)
    total = torch.empty(n_k, dtype=torch.int64, device=dev)
    last = torch.empty(n_k, dtype=torch.int32, device=dev)
    plan = torch.empty((n_k, N), dtype=torch.int32, device=dev)
    plan_mem = torch.empty(n_k, dtype=torch.int64, device=dev)
    first = torch.empty(1, dtype=torch.int32, device=dev)
    limit = 1 << 40                               # per-device parameter memory; the sweep ends at k = 186
    times = {}
    # the chain batch spread over eight workgroups per problem, and (these tables are sparse: a third of the slots
    # are valid layouts) all problems through the segmented route
    for name, kind in (("eight_workgroups_each", rh.WS_MINPLUS_CHAIN), ("segmented", rh.WS_MINPLUS_CHAIN_SEGMENTED)):
        ws_bytes = rh.rh_workspace_size(kind, n_k, N, Kp)
        ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None

        def run():
            rh.rh_mask_replicated(N, Kp, n_k, k0, c, pb, repl, cm)
            rh.rh_minplus_chain(n_k, N, Kp, cm, N * Kp, R, 0, arg, None, total, last, ws)
            rh.rh_backtrack(n_k, N, Kp, arg, last, plan)
            rh.rh_plan_memory(n_k, N, Kp, plan, mem, total, limit, plan_mem, first)

        times[name] = _best_ms(run, reps=2)
        del ws
    t = times["segmented"]
    cells = n_k * (N - 1) * Kp * Kp
    return {"k_values": n_k, "k0": k0, "limit_bytes": limit, "first_feasible_offset": int(first.item()),
            "sweep_ms": t, "sweep_method": "segmented chains",
            "sweep_ms_eight_workgroups_each": times["eight_workgroups_each"], "cells_per_s": cells / (t * 1e-3),
            "shared_table_gbps": cells * 8 / (t * 1e-3) / 1e9}


def _fused_rows(g, dev):
    """The chain DP that computes resharding times per cell (no tables in memory): the graph on the 11
    two-dimensional power-of-two shapes of its 1024-device mesh, once each and cycled to 256 problems."""
    N, Kp = g["N"], g["Kp"]
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    K, osp, isp = to(g["K"]), to(g["out_spec"].view(np.int32)), to(g["in_spec"].view(np.int32))
    dims, eb = to(g["dims"]), to(g["elem_bytes"])
    n_dev = g["m"][0] * g["m"][1]
    shapes = [(1 << k, n_dev >> k) for k in range(n_dev.bit_length())]
    out = {"mesh_shapes": len(shapes)}
    whole = {}                                    # totals of the whole-chain kernel per batch size
    for B in (1, len(shapes), 256):
        meshes = [rh.Mesh.make(shapes[(p + len(shapes) // 2) % len(shapes)], g["bw_bytes_per_us"], g["alpha_ns"])
                  for p in range(min(B, len(shapes)))]
        c = to(g["c"][None]).repeat(B, 1, 1).contiguous()     # node costs of the reference mesh for every problem
        arg = torch.empty((B, N - 1, Kp), dtype=torch.int16, device=dev)
        total = torch.empty(B, dtype=torch.int64, device=dev)
        last = torch.empty(B, dtype=torch.int32, device=dev)
        t = _best_ms(lambda: rh.rh_minplus_chain_specs(B, N, Kp, meshes, c, N * Kp, K, osp, isp, dims, eb, arg, None,
                                                       total, last), reps=2)
        cells = B * (N - 1) * Kp * Kp
        out[f"B{B}"] = {"ms": t, "cells_per_s": cells / (t * 1e-3), "tables_not_stored_gb": cells * 8 / 1e9}
        whole[B] = [int(x) for x in total.tolist()]
    # the segmented route with every table entry computed from the spec words (no table in memory either)
    for B in (1, len(shapes)):
        meshes = [rh.Mesh.make(shapes[(p + len(shapes) // 2) % len(shapes)], g["bw_bytes_per_us"], g["alpha_ns"])
                  for p in range(B)]
        c = to(g["c"][None]).repeat(B, 1, 1).contiguous()
        arg = torch.empty((B, N - 1, Kp), dtype=torch.int16, device=dev)
        total = torch.empty(B, dtype=torch.int64, device=dev)
        last = torch.empty(B, dtype=torch.int32, device=dev)
        ws = torch.empty(rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SPECS, B, N, Kp), dtype=torch.uint8, device=dev)
        t = _best_ms(lambda: rh.rh_minplus_chain_specs(B, N, Kp, meshes, c, N * Kp, K, osp, isp, dims, eb, arg, None,
                                                       total, last, ws), reps=3)
        out[f"B{B}_segmented_from_specs_ms"] = t
        seg_totals = [int(x) for x in total.tolist()]
        del ws
    # the same 11 mesh shapes by the other route: build every mesh's tables, then the segmented chains
    B = len(shapes)
    meshes = [rh.Mesh.make(shapes[(p + B // 2) % B], g["bw_bytes_per_us"], g["alpha_ns"]) for p in range(B)]
    c = to(g["c"][None]).repeat(B, 1, 1).contiguous()
    R = torch.empty((B, N - 1, Kp, Kp), dtype=torch.int64, device=dev)
    arg = torch.empty((B, N - 1, Kp), dtype=torch.int16, device=dev)
    total = torch.empty(B, dtype=torch.int64, device=dev)
    last = torch.empty(B, dtype=torch.int32, device=dev)
    ws = torch.empty(rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SEGMENTED, B, N, Kp), dtype=torch.uint8, device=dev)

    def with_tables():
        for p in range(B):
            rh.rh_build_reshard(meshes[p], N - 1, Kp, K, osp, isp, dims, eb, R[p])
        rh.rh_minplus_chain(B, N, Kp, c, N * Kp, R, (N - 1) * Kp * Kp, arg, None, total, last, ws)

    out["B11_tables_then_segmented_chains_ms"] = _best_ms(with_tables, reps=2)
    out["B11_totals_ns"] = [int(x) for x in total.tolist()]
    if out["B11_totals_ns"] != seg_totals:
        raise RuntimeError("the two routes over the 11 mesh shapes disagree")
    # problem p of every batch is the graph on mesh shape p mod 11: the whole-chain kernel must agree with both
    for Bw, got in whole.items():
        if got != [seg_totals[p % B] for p in range(Bw)]:
            raise RuntimeError(f"the whole-chain kernel on {Bw} problems disagrees with the segmented routes")
    return out


def _graph_rows(g, dev):
    N, Kp = g["N"], g["Kp"]
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    mesh = rh.Mesh.make(g["m"], g["bw_bytes_per_us"], g["alpha_ns"])
    K, osp, isp = to(g["K"]), to(g["out_spec"].view(np.int32)), to(g["in_spec"].view(np.int32))
    dims, eb, c = to(g["dims"]), to(g["elem_bytes"]), to(g["c"][None])
    R = torch.empty((N - 1, Kp, Kp), dtype=torch.int64, device=dev)
    arg = torch.empty((1, N - 1, Kp), dtype=torch.int16, device=dev)
    total = torch.empty(1, dtype=torch.int64, device=dev)
    last = torch.empty(1, dtype=torch.int32, device=dev)
    plan = torch.empty((1, N), dtype=torch.int32, device=dev)
    t_build = _best_ms(lambda: rh.rh_build_reshard(mesh, N - 1, Kp, K, osp, isp, dims, eb, R))
    scratch = torch.empty_like(R)
    t_write = _best_ms(lambda: device_fill.stream_write(scratch))   # plain write-only kernel, same number of bytes
    del scratch
    ws_bytes = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, 1, N, Kp)
    ws = torch.empty(ws_bytes, dtype=torch.uint8, device=dev) if ws_bytes else None
    t_chain = _best_ms(lambda: rh.rh_minplus_chain(1, N, Kp, c, N * Kp, R, (N - 1) * Kp * Kp, arg, None, total, last,
                                                   ws))
    t_back = _best_ms(lambda: rh.rh_backtrack(1, N, Kp, arg, last, plan))
    table_total = int(total.item())
    # tables and chain in one go, against the segmented route that computes the entries from the spec words
    def tables_then_chain():
        rh.rh_build_reshard(mesh, N - 1, Kp, K, osp, isp, dims, eb, R)
        rh.rh_minplus_chain(1, N, Kp, c, N * Kp, R, (N - 1) * Kp * Kp, arg, None, total, last, ws)
    t_both = _best_ms(tables_then_chain)
    ws_s = torch.empty(rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SPECS, 1, N, Kp), dtype=torch.uint8, device=dev)
    t_specs = _best_ms(lambda: rh.rh_minplus_chain_specs(1, N, Kp, [mesh], c, N * Kp, K, osp, isp, dims, eb, arg, None,
                                                         total, last, ws_s))
    if int(total.item()) != table_total:
        raise RuntimeError("the chain from specs disagrees with the chain over the tables")
    del ws_s
    cells = (N - 1) * Kp * Kp
    extra = {"memory_sweep": _memory_sweep_rows(g, R, dev), "fused_no_tables": _fused_rows(g, dev)} if Kp == 256 else {}
    return {**extra, "N": N, "K": Kp, "mesh": list(g["m"]), "total_ns": int(total.item()),
            "reshard_ms": t_build, "reshard_write_gbps": cells * 8 / (t_build * 1e-3) / 1e9,
            "plain_write_kernel_gbps": cells * 8 / (t_write * 1e-3) / 1e9,
            "chain_method": "segments: matrices, boundary vectors, batched sweep" if ws_bytes else "one workgroup",
            "chain_ms": t_chain, "chain_cells_per_s": cells / (t_chain * 1e-3),
            "chain_hbm_gbps": cells * 8 * (1 + 1.25 / Kp) / (t_chain * 1e-3) / 1e9,
            "reshard_then_chain_ms": t_both, "chain_from_specs_segmented_ms": t_specs,
            "backtrack_ms": t_back}


def _stage_rows(dev):
    w = syn.STAGE_PARTITION
    L, S, M, K = w["L"], w["S"], w["seg_ops"], w["seg_K"]
    c = torch.empty((L, M, K), dtype=torch.int64, device=dev)
    R = torch.empty((L, M - 1, K, K), dtype=torch.int64, device=dev)
    device_fill.fill_random_chain(c, R, 0, w["seg_c_range"], w["seg_r_range"], c_lo=w["seg_c_lo"])
    arg = torch.empty((L, M - 1, K), dtype=torch.int16, device=dev)
    seg = torch.empty(L, dtype=torch.int64, device=dev)
    last = torch.empty(L, dtype=torch.int32, device=dev)
    t_seg = _best_ms(lambda: rh.rh_minplus_chain(L, M, K, c, M * K, R, (M - 1) * K * K, arg, None, seg, last))
    bott = torch.empty((1, S), dtype=torch.int64, device=dev)
    cut = torch.empty((1, S, L + 1), dtype=torch.int32, device=dev)
    bounds = torch.empty((1, S + 1), dtype=torch.int32, device=dev)
    ws = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP, 1, L, S), dtype=torch.uint8, device=dev)
    cost = seg.reshape(1, L)
    t_dp = _best_ms(lambda: rh.rh_stage_dp(1, L, S, cost, bott, cut, S, bounds, ws))
    cells = sum((L - s + 1) * (L - s + 2) // 2 for s in range(2, S + 1))      # (i, j) pairs with s-1 <= i < j <= L
    # 256 chains of segments at once (one per candidate mesh, say): costs of problem p are problem 0's rotated by p
    Bm = 256
    costs = torch.stack([torch.roll(seg, p) for p in range(Bm)])
    bott_m = torch.empty((Bm, S), dtype=torch.int64, device=dev)
    cut_m = torch.empty((Bm, S, L + 1), dtype=torch.int32, device=dev)
    ws_m = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP, Bm, L, S), dtype=torch.uint8, device=dev)
    t_dp_m = _best_ms(lambda: rh.rh_stage_dp(Bm, L, S, costs, bott_m, cut_m, 0, None, ws_m))
    del costs, bott_m, cut_m, ws_m
    # the same partition for exactly S stages with boundary transfers and a tolerance of half a stage
    xfer = torch.from_numpy(syn.uniform_at(syn.stream_seed(syn.BASE_SEED, 0, 7), np.arange(L + 1, dtype=np.uint64),
                                           50000)[None]).to(dev)
    wb = torch.empty(1, dtype=torch.int64, device=dev)
    ws2 = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP_WINDOW, 1, L, S), dtype=torch.uint8, device=dev)
    t_win = _best_ms(lambda: rh.rh_stage_dp_window(1, L, S, cost, xfer, 1, 2, wb, cut, bounds, ws2))
    interval = _interval_rows(dev, L, S, K)
    return {"L": L, "S": S, "segment_chain": {"ops": M, "K": K}, "segment_chains_ms": t_seg,
            "interval_stage_times": interval,
            "stage_dp_ms": t_dp, "stage_dp_us_per_stage_count": t_dp * 1e3 / S,
            "stage_dp_256_problems_ms": t_dp_m, "stage_dp_256_problems_per_s": Bm / (t_dp_m * 1e-3),
            "stage_dp_method": "bisection on the monotone crossing point (exact, O(S L log L)); one workgroup per "
                               "problem, bound by one compute unit's vector ALU",
            "stage_dp_full_scan_cells_not_visited": cells,
            "bottleneck_ns_at_S": int(bott[0, S - 1].item()),
            "window_eps_half_with_transfers_ms": t_win, "window_bottleneck_ns": int(wb.item())}


def _interval_rows(dev, L, S, K):
    """Stage time = the stage's own best plan: every segment an operator with K boundary strategies; the table of
    all L(L+1)/2 candidate stages, then the stage search over it."""
    c = torch.empty((1, L, K), dtype=torch.int64, device=dev)
    R = torch.empty((1, L - 1, K, K), dtype=torch.int64, device=dev)
    device_fill.fill_random_chain(c, R, 11, 100_000, 200_000)
    ldT = L + 2 - (L & 1)
    T = torch.empty((1, L, ldT), dtype=torch.int64, device=dev)
    t_tab = _best_ms(lambda: rh.rh_interval_costs(1, L, K, c, R, ldT, T))
    cells_tab = sum(L - 1 - i for i in range(L)) * K * K
    # the same table put together from blocks of 128 operators (the call with its workspace)
    T_rows = T.clone()
    ws_b = torch.empty(rh.rh_workspace_size(rh.WS_INTERVAL_COSTS, 1, L, K), dtype=torch.uint8, device=dev)
    t_blk = _best_ms(lambda: rh.rh_interval_costs(1, L, K, c, R, ldT, T, ws_b)) if ws_b.numel() else None
    if t_blk is not None and not torch.equal(T[:, :, :L + 1], T_rows[:, :, :L + 1]):
        raise RuntimeError("the table from blocks differs from the table row by row")
    del T_rows, ws_b
    bott = torch.empty((1, S), dtype=torch.int64, device=dev)
    cut = torch.empty((1, S, L + 1), dtype=torch.int32, device=dev)
    bounds = torch.empty((1, S + 1), dtype=torch.int32, device=dev)
    ws = torch.empty(rh.rh_workspace_size(rh.WS_STAGE_DP_INTERVAL, 1, L, S), dtype=torch.uint8, device=dev)
    t_dp = _best_ms(lambda: rh.rh_stage_dp_interval(1, L, S, ldT, T, bott, cut, S, bounds, ws))
    cells_dp = sum((L - s + 1) * (L - s + 2) // 2 for s in range(2, S + 1))
    # the same with no stage longer than four times the balanced length (Sec. 5.2 keeps operators near their stage)
    max_len = 4 * L // S
    t_tab_b = _best_ms(lambda: rh.rh_interval_costs_banded(1, L, K, max_len, c, R, ldT, T))
    cells_tab_b = sum(min(L - 1 - i, max_len - 1) for i in range(L)) * K * K
    T_rows = T.clone()
    ws_b = torch.empty(rh.rh_workspace_size(rh.WS_INTERVAL_COSTS, 1, L, K), dtype=torch.uint8, device=dev)
    t_blk_b = _best_ms(lambda: rh.rh_interval_costs_banded(1, L, K, max_len, c, R, ldT, T, ws_b)) if ws_b.numel() else None
    if t_blk_b is not None and not torch.equal(T[:, :, :L + 1], T_rows[:, :, :L + 1]):
        raise RuntimeError("the limited table from blocks differs from the limited table row by row")
    del T_rows, ws_b
    t_dp_b = _best_ms(lambda: rh.rh_stage_dp_interval_banded(1, L, S, max_len, ldT, T, bott, cut, S, bounds, ws))
    banded = {"max_len": max_len, "table_ms": t_tab_b, "table_from_blocks_ms": t_blk_b, "table_cells": cells_tab_b,
              "table_cells_per_s": cells_tab_b / (t_tab_b * 1e-3), "search_ms": t_dp_b,
              "bottleneck_ns_at_S": int(bott[0, S - 1].item())}
    rh.rh_interval_costs(1, L, K, c, R, ldT, T)
    rh.rh_stage_dp_interval(1, L, S, ldT, T, bott, cut, S, bounds, ws)
    # the plans of the S chosen stages, all at once
    arg = torch.empty((1, L - 1, K), dtype=torch.int16, device=dev)
    st_total = torch.empty((1, S), dtype=torch.int64, device=dev)
    st_last = torch.empty((1, S), dtype=torch.int32, device=dev)
    plan = torch.empty((1, L), dtype=torch.int32, device=dev)
    t_plans = _best_ms(lambda: rh.rh_stage_plans(1, L, K, S, bounds, c, R, arg, st_total, st_last, plan))
    if int(st_total.max().item()) != int(bott[0, S - 1].item()) or int(plan.min().item()) < 0:
        raise RuntimeError("the stages' own plans do not reach the bottleneck the search found")
    return {"K": K, "stages_of_limited_length": banded, "stage_plans_ms": t_plans,
            "table_ms": t_tab, "table_cells": cells_tab, "table_cells_per_s": cells_tab / (t_tab * 1e-3),
            "table_from_blocks_ms": t_blk,
            "table_f64_lane_ops_per_s": 2 * cells_tab / (t_tab * 1e-3),
            "search_ms": t_dp, "search_cells": cells_dp, "search_cells_per_s": cells_dp / (t_dp * 1e-3),
            "search_table_read_gbps": cells_dp * 8 / (t_dp * 1e-3) / 1e9,
            "bottleneck_ns_at_S": int(bott[0, S - 1].item())}


def _cone_rows(dev, n_cones=1024, K=64):
    """Cones (one root, up to four chain branches of up to six operators): branch batch through the chain DP,
    merge at the roots, backtrack every branch."""
    pk = wc.pack(wc.random_cones(n_cones, K), K)
    c, R = torch.from_numpy(pk["c"]).to(dev), torch.from_numpy(pk["R"]).to(dev)
    Bb, N, Kp = pk["c"].shape
    start, c_root = torch.from_numpy(pk["branch_start"]).to(dev), torch.from_numpy(pk["c_root"]).to(dev)
    arg = torch.empty((Bb, N - 1, Kp), dtype=torch.int16, device=dev)
    w = torch.empty((Bb, Kp), dtype=torch.int64, device=dev)
    tot_b = torch.empty(Bb, dtype=torch.int64, device=dev)
    last_b = torch.empty(Bb, dtype=torch.int32, device=dev)
    table = torch.empty((n_cones, Kp), dtype=torch.int64, device=dev)
    total = torch.empty(n_cones, dtype=torch.int64, device=dev)
    choice = torch.empty(n_cones, dtype=torch.int32, device=dev)
    branch_last = torch.empty(Bb, dtype=torch.int32, device=dev)
    plan = torch.empty((Bb, N), dtype=torch.int32, device=dev)

    def run():
        rh.rh_minplus_chain(Bb, N, Kp, c, N * Kp, R, (N - 1) * Kp * Kp, arg, w, tot_b, last_b)
        rh.rh_cone_merge(n_cones, Bb, Kp, start, w, c_root, table, total, choice, branch_last)
        rh.rh_backtrack(Bb, N, Kp, arg, branch_last, plan)

    t = _best_ms(run)
    return {"cones": n_cones, "branches": Bb, "K": K, "ops_per_branch_padded": N, "chain_merge_backtrack_ms": t,
            "cones_per_s": n_cones / (t * 1e-3)}


def _tree_rows(dev, n=4096, K=64, B=8):
    """One in-tree of operators (inner nodes join up to four inputs) searched for B problems at once."""
    from .workloads import trees
    parent = trees.random_tree(n, max_fan_in=4, chain_bias=0.7)
    c, R = trees.random_tree_costs(parent, K)
    tp = rh.TreePlan(parent, dev)
    dc = torch.from_numpy(c[None]).to(dev).repeat(B, 1, 1).contiguous()
    dR = torch.from_numpy(R).to(dev)
    arg = torch.empty((B, n - 1, K), dtype=torch.int16, device=dev)
    w = torch.empty((B, n, K), dtype=torch.int64, device=dev)
    total = torch.empty(B, dtype=torch.int64, device=dev)
    choice = torch.empty(B, dtype=torch.int32, device=dev)
    plan = torch.empty((B, n), dtype=torch.int32, device=dev)
    t = _best_ms(lambda: rh.rh_tree_dp(B, K, tp, dc, n * K, dR, 0, arg, w, total, choice, plan))
    runs = tp.host["run_last"][:tp.n_runs] - tp.host["run_first"][:tp.n_runs] + 1
    return {"nodes": n, "K": K, "problems": B, "depth": trees.depth(parent), "runs": tp.n_runs, "rounds": tp.n_rounds,
            "longest_run": int(runs.max()), "dp_and_plan_ms": t, "cells_per_s": B * (n - 1) * K * K / (t * 1e-3),
            "total_ns": int(total[0].item())}


def measure(dev="cuda:0"):
    return {"moe_shaped_graph": _graph_rows(graphs.moe_chain(), dev),
            "gpt_like_chain": _graph_rows(graphs.gpt_chain(), dev),
            "stage_partition": _stage_rows(dev),
            "cones": _cone_rows(dev),
            "in_tree": _tree_rows(dev)}
