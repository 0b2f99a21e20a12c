#!/usr/bin/env python3
"""Benchmark of plan scoring on one MI355X.

A step is one pass of the scoring path over the batched-random-chains workload
(B=4096 independent chains, N=512 operators, K=128 candidates; node costs
uniform [0,1e6), edge tables uniform [0,1e7) with zero diagonal, one SplitMix64
stream per problem): rh_minplus_chain over all problems, then rh_backtrack.
The cost tables are generated on the device before the timed region and stay
resident in HBM (274.3 GB of edge tables).  The metric is min-plus cell
relaxations per second (one cell = one (a, b) pair of one edge of one problem).

The same run also reports, outside the timed steps: the roofline of the chain
kernel from per-launch HIP-event times, the CPU oracle on the host cores on a
sample of the same problems, and the other rows of the path on their own
workloads (reshard-table generation + chain + backtrack on the MoE-shaped
graph, the pipeline-stage DP with per-segment chains).

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import gc
import hashlib
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--problems", type=int, default=0, help="override B (debugging only; 0 = the workload's 4096)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-other-rows", action="store_true")
    ap.add_argument("--rows-only", action="store_true",
                    help="only time the other rows of the path (for profiling them); prints their JSON")
    return ap.parse_args()


def kernel_source_hash() -> str:
    src = os.path.join(ROOT, "paper_2302_08141_amd", "csrc", "chain_dp.hip")
    return hashlib.sha256(open(src, "rb").read()).hexdigest()[:16]


def recorded_traffic(kernel_hash: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if it was taken on this kernel source."""
    path = os.path.join(ROOT, "profiles", "chain_coop_kernel_batched_chains_pmc.md")
    if not os.path.exists(path):
        return None
    text = open(path).read()
    h = re.search(r"kernel_source_sha256_16:\s*([0-9a-f]+)", text)
    t = re.search(r"traffic_bytes_per_launch:\s*([0-9.eE+]+)", text)
    if not h or not t or h.group(1) != kernel_hash:
        return None
    return float(t.group(1))


def host_threads() -> int:
    n = len(os.sched_getaffinity(0))
    env = os.environ.get("OMP_NUM_THREADS")
    if env and env.isdigit() and int(env) > 0:
        n = min(n, int(env))
    return max(n, 1)


def cpu_baseline(c, R, B, N, K, gpu_total, gpu_last, gpu_plan, sample_problems=4096, batch=64, single=256):
    """The oracle as it stands, on the host cores, on the first `sample_problems` problems of the batch
    (copied back from HBM in slices; copies are not timed), then on `single` of them with one thread.  Its totals,
    last strategies and plans are compared with what the timed GPU steps left behind: a mismatch ends the run."""
    import numpy as np
    import oracle
    threads = host_threads()
    n = min(sample_problems, B)
    spent, done, bad = 0.0, 0, []
    g_total, g_last, g_plan = gpu_total[:n].cpu().numpy(), gpu_last[:n].cpu().numpy(), gpu_plan[:n].cpu().numpy()
    while done < n:
        m = min(batch, n - done)
        hc = c[done:done + m].cpu().numpy()
        hR = R[done:done + m].cpu().numpy()
        t0 = time.perf_counter()
        arg, _, total, last = oracle.chain(hc, hR, nthreads=threads)
        plan = oracle.backtrack(arg, last)
        spent += time.perf_counter() - t0
        ok = (total == g_total[done:done + m]) & (last == g_last[done:done + m]) & \
             (plan == g_plan[done:done + m]).all(axis=1)
        bad += [done + int(i) for i in np.nonzero(~ok)[0]]
        done += m
        del hc, hR
    if bad:
        print(f"PARITY FAILURE: the GPU's total, last or plan differs from the oracle's on problems {bad[:16]} "
              f"({len(bad)} of {n})", file=sys.stderr)
        sys.exit(1)
    cells = n * (N - 1) * K * K
    n1 = min(single, n)
    hc, hR = c[:n1].cpu().numpy(), R[:n1].cpu().numpy()
    t0 = time.perf_counter()
    arg, _, total, last = oracle.chain(hc, hR, nthreads=1)
    oracle.backtrack(arg, last)
    spent1 = time.perf_counter() - t0
    return {"value": cells / spent, "unit": "cells/s", "cores": threads, "kind": "oracle",
            "sample": f"first {n} of {B} problems (N={N}, K={K}), {spent:.1f} s of oracle time, "
                      f"one problem per thread",
            "single_thread_value": n1 * (N - 1) * K * K / spent1,
            "single_thread_sample": f"first {n1} problems, {spent1:.1f} s on one thread",
            "parity_checked_problems": n}


def cpu_other_rows():
    """The oracle as it stands on bounded samples of the other workloads (part of the CPU-baseline leg): the
    unit-counting reshard builder on edges of the MoE-shaped graph, the stage search on the stage-partition chain, the
    interval table on a prefix of it."""
    import numpy as np
    import oracle
    from paper_2302_08141_amd.workloads import graphs, synthetic as syn
    out = {}
    g = graphs.moe_chain()
    e0, ne = 85, 8                                    # eight edges of the second layer
    sl = slice(e0, e0 + ne + 1)
    t0 = time.perf_counter()
    oracle.build_reshard(g["m"], g["bw_bytes_per_us"], g["alpha_ns"], g["K"][sl], g["out_spec"][sl], g["in_spec"][sl],
                         g["dims"][e0:e0 + ne], g["elem_bytes"][e0:e0 + ne])
    dt = time.perf_counter() - t0
    out["moe_reshard_builder"] = {"ms_per_edge": dt * 1e3 / ne, "edges_timed": ne, "of_edges": g["N"] - 1,
                                  "K": g["Kp"], "cores": 1, "kind": "oracle (counts units per device)"}
    w = syn.STAGE_PARTITION
    L, S = w["L"], w["S"]
    cost = syn.segment_costs(0, L, w["lo"], w["hi"])[None]
    threads = host_threads()
    t0 = time.perf_counter()
    oracle.stage_dp(cost, S, s_query=S, nthreads=1)
    dt = time.perf_counter() - t0
    cells = sum((L - s + 1) * (L - s + 2) // 2 for s in range(2, S + 1))
    out["stage_dp"] = {"ms": dt * 1e3, "L": L, "S": S, "max_min_cells_per_s": cells / dt, "cores": 1,
                       "kind": "oracle (full scan)"}
    Ls, K = 512, 64                                   # the interval table of the first 512 segments
    c, R = syn.random_chain_batch([11], Ls, K, 100_000, 200_000)
    t0 = time.perf_counter()
    oracle.interval_costs(c[0], R[0], nthreads=threads)
    dt = time.perf_counter() - t0
    out["interval_table"] = {"ms": dt * 1e3, "L": Ls, "of_L": L, "K": K,
                             "cells_per_s": sum(Ls - 1 - i for i in range(Ls)) * K * K / dt, "cores": threads,
                             "kind": "oracle"}
    return out


def main():
    args = parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2302_08141_amd import binding as rh
    from paper_2302_08141_amd.workloads import device_fill, synthetic as syn

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    rh.lib()
    dev = "cuda:0"
    if args.rows_only:
        from paper_2302_08141_amd import other_rows
        print(json.dumps({"other_rows": other_rows.measure(dev)}))
        return
    w = syn.BATCHED_CHAINS
    B, N, K = (args.problems or w["B"]), w["N"], w["K"]

    need = B * ((N - 1) * K * K * 8 + N * K * 8 + (N - 1) * K * 2 + N * 4 + 16)
    free, _ = torch.cuda.mem_get_info()
    if need > free - (2 << 30):
        print(f"the workload needs {need / 2**30:.1f} GiB resident, {free / 2**30:.1f} GiB are free", file=sys.stderr)
        sys.exit(3)

    c = torch.empty((B, N, K), dtype=torch.int64, device=dev)
    R = torch.empty((B, N - 1, K, K), dtype=torch.int64, device=dev)
    arg = torch.empty((B, N - 1, K), dtype=torch.int16, device=dev)
    total = torch.empty(B, dtype=torch.int64, device=dev)
    last = torch.empty(B, dtype=torch.int32, device=dev)
    plan = torch.empty((B, N), dtype=torch.int32, device=dev)
    # fill in slices so that one launch stays short
    for p0 in range(0, B, 256):
        p1 = min(B, p0 + 256)
        device_fill.fill_random_chain(c[p0:p1], R[p0:p1], p0, w["c_range"], w["r_range"])
    torch.cuda.synchronize()

    def step(events=None):
        if events is not None:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
        rh.rh_minplus_chain(B, N, K, c, N * K, R, (N - 1) * K * K, arg, None, total, last)
        if events is not None:
            e1.record()
            events.append((e0, e1))
        rh.rh_backtrack(B, N, K, arg, last, plan)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = []
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step(events)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    cells = B * (N - 1) * K * K
    ms_per_step = elapsed * 1e3 / args.steps
    value = cells * args.steps / elapsed

    # roofline of the chain kernel: algorithmic bytes per launch / mean launch time (HIP events on the launch stream)
    kern_ms = sum(a.elapsed_time(b) for a, b in events) / len(events)
    bytes_per_cell = 8.0 * (1.0 + 1.25 / K)                 # R once, plus c read and arg written per edge row
    algo_bytes = cells * bytes_per_cell
    achieved = algo_bytes / (kern_ms * 1e-3) / 1e9
    khash = kernel_source_hash()
    roofline = {"bound": "hbm", "kernel": f"chain_coop_kernel<{K},16>", "achieved": achieved, "peak": HBM_PEAK_GBPS,
                "unit": "GB/s", "frac": achieved / HBM_PEAK_GBPS, "traffic": recorded_traffic(khash),
                "algorithmic_bytes_per_launch": algo_bytes, "kernel_ms": kern_ms}

    out = {"metric": "min-plus cell relaxations/sec (K^2 per edge, batched)", "value": value, "unit": "cells/s",
           "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
           "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int64", "data": "synthetic",
           "config": {"workload": f"batched random chains: B={B} N={N} K={K}, c~U[0,1e6) R~U[0,1e7) zero diagonal, "
                                  f"all tables resident in HBM; step = rh_minplus_chain + rh_backtrack",
                      "B": B, "N": N, "K": K, "seed": syn.BASE_SEED},
           "achieved_hbm_gbps": achieved, "roofline": roofline}

    # yardsticks on the same box: a plain read-only stream over part of R and a plain copy of known size
    sink = torch.zeros(1, dtype=torch.int64, device=dev)
    probe = R[: min(B, 512)]
    copy_src = R[: min(B, 64)]
    copy_dst = torch.empty_like(copy_src)
    rates = {}
    for name, fn, nbytes in (("read", lambda: device_fill.stream_read(probe, sink), probe.numel() * 8),
                             ("read_wide", lambda: device_fill.stream_read(probe, sink, blocks=2048, wide=True),
                              probe.numel() * 8),
                             ("read_slices", lambda: device_fill.stream_read(probe, sink, blocks=2048, slices=True),
                              probe.numel() * 8),
                             ("read_slices_256", lambda: device_fill.stream_read(probe, sink, blocks=256, slices=True),
                              probe.numel() * 8),
                             ("copy", lambda: device_fill.stream_copy(copy_dst, copy_src), copy_src.numel() * 8)):
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(); fn(); e1.record()
            torch.cuda.synchronize()
            t = e0.elapsed_time(e1)
            best = t if best is None or t < best else best
        rates[name] = nbytes / (best * 1e-3) / 1e9
    del copy_dst
    rates["read"] = max(rates["read"], rates.pop("read_wide"), rates.pop("read_slices"),
                        rates.pop("read_slices_256"))
    out["streaming_read_ceiling_gbps"] = rates["read"]
    out["streaming_copy_gbps_read_plus_write"] = 2 * rates["copy"]
    out["roofline"]["frac_of_measured_read_ceiling"] = achieved / rates["read"]
    out["roofline"]["copy_kernel_bytes_each_way"] = copy_src.numel() * 8

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(c, R, B, N, K, total, last, plan)
        out["parity_checked_problems"] = out["cpu_baseline"]["parity_checked_problems"]
        out["gpu_over_cpu"] = value / out["cpu_baseline"]["value"]
        out["cpu_baseline"]["other_rows"] = cpu_other_rows()

    # the other rows need room of their own (one of them holds the tables of 11 meshes): every view of R goes too
    del c, R, arg, plan, probe, copy_src, fn
    gc.collect()
    torch.cuda.empty_cache()
    if not args.no_other_rows:
        from paper_2302_08141_amd import other_rows
        out["other_rows"] = other_rows.measure(dev)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
