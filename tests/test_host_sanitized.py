"""The library's host side (argument checks, the tree planner, workspace sizes, the sizing rule of the
several-workgroups route) once more in a build whose host code runs under the address and undefined-behaviour
sanitizers (CPU only; device code is compiled as usual and never launched here).

The sanitizer runtime has to be in the process before Python starts, so the checks run in a child process that
preloads it in front of whatever the environment preloads already; RHINO_LIBRARY points the binding at the
instrumented build.  Output arrays have exactly the sizes the header documents, so a write one element past an
array aborts the child.
"""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r'''
import ctypes, sys
import numpy as np
from paper_2302_08141_amd import binding as rh
from paper_2302_08141_amd.workloads import trees
L = rh.lib()
assert L._name.endswith("librhino_hostsan.so"), L._name
hp = lambda a: a.ctypes.data_as(ctypes.c_void_p)

# the tree planner: arrays of exactly the documented sizes, trees from a single node to bushy and path-like ones
for seed in range(40):
    n = [1, 2, 3, 9, 40, 200, 1000][seed % 7]
    parent = trees.random_tree(n, max_fan_in=1 + seed % 5, chain_bias=[0.0, 0.5, 0.9][seed % 3], seed=seed)
    run_first, run_last, child_list = (np.full(n, -7, np.int32) for _ in range(3))
    round_start, child_start = (np.full(n + 1, -7, np.int32) for _ in range(2))
    n_runs = ctypes.c_int32(-1)
    rounds = L.rh_tree_plan(n, hp(parent), hp(run_first), hp(run_last), hp(round_start), hp(child_start),
                            hp(child_list), ctypes.byref(n_runs))
    assert rounds >= 1 and 1 <= n_runs.value <= n, (seed, rounds, n_runs.value)
    assert round_start[0] == 0 and round_start[rounds] == n_runs.value
    covered = np.zeros(n, np.int64)
    for u in range(n_runs.value):
        covered[run_first[u]:run_last[u] + 1] += 1
    assert (covered == 1).all()
# parent arrays that are no in-trees are refused, not walked
for bad in ([-1, -1], [1, 0, -1], [2, 2, 1], [5, -1]):
    b = np.array(bad, np.int32); n = len(bad)
    o = [np.zeros(n + 1, np.int32) for _ in range(5)]
    assert L.rh_tree_plan(n, hp(b), *[hp(a) for a in o], ctypes.byref(ctypes.c_int32())) < 0

# workspace sizes and the sizing rule over their whole argument ranges (corners included)
for which in range(8):
    for B in (-1, 0, 1, 2, 3, 32, 33, 64, 65, 4096, 65535, 1 << 30):
        for N in (-5, 0, 1, 63, 64, 127, 128, 511, 512, 4096, 16384, 16385, 1 << 30):
            for K in (-1, 0, 1, 15, 16, 48, 64, 128, 256, 512, 1024, 2048):
                rh.rh_workspace_size(which, B, N, K)
for which in (0, 3, 4, 5, 6):                      # the planners behind the sizes, over the whole range of lengths
    for N in list(range(1, 700)) + list(range(700, 16386, 37)):
        for K in (64, 128, 256):
            for B in (1, 2, 3, 32):
                rh.rh_workspace_size(which, B, N, K if which != 3 else min(N, 64))
for B in (-3, 0, 1, 31, 32, 33, 64, 65, 1 << 30):
    for cus in (-1, 0, 1, 8, 104, 256, 304, 1 << 30):
        assert rh.rh_gang_workgroups(B, cus) in (0, 4, 8)

# every entry point's argument checks with NULL buffers: an error code comes back, nothing is dereferenced
N_ = None
assert L.rh_build_reshard(None, 1, 64, N_, N_, N_, N_, N_, N_, N_) < 0
m = rh.Mesh.make((4, 8), (1000, 1000), (0, 0))
assert L.rh_build_reshard(ctypes.byref(m), 3, 64, N_, N_, N_, N_, N_, N_, N_) < 0
assert L.rh_build_reshard(ctypes.byref(m), -1, 64, N_, N_, N_, N_, N_, N_, N_) < 0
assert L.rh_minplus_chain(4, 8, 64, N_, 512, N_, 0, N_, N_, N_, N_, N_, 0, N_) < 0
assert L.rh_minplus_chain(4, 0, 64, N_, 512, N_, 0, N_, N_, N_, N_, N_, 0, N_) < 0
assert L.rh_minplus_chain(4, 8, 48, N_, 512, N_, 0, N_, N_, N_, N_, N_, 0, N_) < 0
assert L.rh_minplus_chain_specs(2, 8, 64, 1, ctypes.byref(m), N_, 512, N_, N_, N_, N_, N_, N_, N_, N_, N_, N_, 0, N_) < 0
assert L.rh_minplus_chain_specs(2, 8, 64, 0, N_, N_, 512, N_, N_, N_, N_, N_, N_, N_, N_, N_, N_, 0, N_) < 0
assert L.rh_backtrack(2, 8, 64, N_, N_, N_, N_) < 0
assert L.rh_stage_dp(1, 8, 9, N_, N_, N_, 0, N_, N_, 0, N_) < 0
assert L.rh_stage_dp(1, 8, 4, N_, N_, N_, 0, N_, N_, 0, N_) < 0
assert L.rh_stage_dp_window(1, 8, 4, N_, N_, 1, 0, N_, N_, N_, N_, 0, N_) < 0
assert L.rh_stage_dp_window_static(1, 8, 4, N_, N_, 1, 2, N_, N_, N_, N_) < 0
assert L.rh_interval_costs(1, 8, 64, N_, N_, 10, N_, N_, 0, N_) < 0
assert L.rh_interval_costs_banded(1, 8, 64, 0, N_, N_, 10, N_, N_, 0, N_) < 0
assert L.rh_stage_dp_interval(1, 8, 4, 10, N_, N_, N_, 0, N_, N_, 0, N_) < 0
assert L.rh_stage_dp_interval_banded(1, 8, 4, 3, 10, N_, N_, N_, 0, N_, N_, 0, N_) < 0
assert L.rh_stage_plans(1, 8, 64, 2, N_, N_, N_, N_, N_, N_, N_, N_) < 0
assert L.rh_cone_merge(2, 3, 64, N_, N_, N_, N_, N_, N_, N_, N_) < 0
rs = np.array([0, 1], np.int32)
assert L.rh_tree_dp(1, 4, 64, 1, 1, hp(rs), N_, N_, N_, N_, N_, N_, 256, N_, 0, N_, N_, N_, N_, N_, N_) < 0
assert L.rh_tree_dp(1, 4, 64, 2, 1, hp(rs), N_, N_, N_, N_, N_, N_, 256, N_, 0, N_, N_, N_, N_, N_, N_) < 0
assert L.rh_mask_replicated(8, 64, 2, 0, N_, N_, N_, N_, N_) < 0
assert L.rh_plan_memory(2, 8, 64, N_, N_, N_, 1, N_, N_, N_) < 0
assert L.rh_check_costs(N_, 10, N_, N_) < 0
for code in range(-12, 3):
    assert isinstance(rh.strerror(code), str)
print("host checks ok")
'''


def test_host_side_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    from paper_2302_08141_amd import build as hip_build
    lib = hip_build.build_host_sanitized(str(tmp_path / "librhino_hostsan.so"))
    runtime = hip_build.host_sanitizer_runtime()
    assert os.path.isabs(runtime) and os.path.exists(runtime), "the compiler has no shared AddressSanitizer runtime"
    env = dict(os.environ)
    env["RHINO_LIBRARY"] = lib
    env["LD_PRELOAD"] = ":".join(x for x in (runtime, env.get("LD_PRELOAD", "")) if x)
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    r = subprocess.run([sys.executable, "-c", CHILD], cwd=ROOT, env=env, stdout=subprocess.PIPE,
                       stderr=subprocess.STDOUT, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-4000:]
    assert "host checks ok" in r.stdout and "ERROR: AddressSanitizer" not in r.stdout and "runtime error" not in r.stdout
