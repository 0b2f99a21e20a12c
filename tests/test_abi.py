"""The C-ABI library loads without a GPU and exports every entry point the header declares."""
import ctypes
import os
import re

from paper_2302_08141_amd import binding as rh

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "rhino.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rh_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    names = declared_functions()
    assert {"rh_build_reshard", "rh_minplus_chain", "rh_backtrack", "rh_stage_dp", "rh_workspace_size",
            "rh_strerror", "rh_version", "rh_check_costs"} <= set(names)
    lib = ctypes.CDLL(rh.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n


def test_header_is_plain_c(tmp_path):
    # the boundary is a C ABI: the header compiles as C99 on its own, and a C program that names every entry point
    # links against the library (no device is touched: only host-side calls are made)
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    assert gcc is not None
    hdr = os.path.join(ROOT, "include", "rhino.h")
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c", hdr],
                   check=True)
    src = tmp_path / "use.c"
    names = declared_functions()
    src.write_text('#include "rhino.h"\n#include <stdio.h>\nint main(void) {\n'
                   + "".join(f"    if ((void*)&{n} == 0) return 2;\n" for n in names)
                   + '    printf("%d %s\\n", rh_version(), rh_strerror(0));\n'
                   + "    return rh_workspace_size(RH_WS_STAGE_DP, 1, 64, 8) > 0 ? 0 : 1;\n}\n")
    exe = tmp_path / "use"
    libdir = os.path.dirname(rh.LIB_PATH)
    subprocess.run([gcc, "-std=c99", "-Wall", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe),
                    "-L", libdir, "-l:" + os.path.basename(rh.LIB_PATH), "-Wl,-rpath," + libdir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) == rh.rh_version() and out[1] == "ok"


def test_host_only_calls():
    assert rh.rh_version() >= 100
    for which in range(8):                                   # no problems: no workspace (and no division by B)
        assert rh.rh_workspace_size(which, 0, 4096, 64) == 0 and rh.rh_workspace_size(which, -1, 4096, 64) == 0
    assert rh.strerror(0) == "ok" and "NULL" in rh.strerror(-1)
    assert rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, 4096, 512, 128) == 0
    # one or two long chains: room for the segment matrices (two thirds + whole), at least a Kp x Kp table each
    one = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, 1, 8192, 256)
    assert one > 3 * 70 * 256 * 256 * 8 and rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, 2, 8192, 256) == 2 * one
    assert rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, 1, 128, 64) > 0
    assert rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, 1, 127, 64) == 0          # too short to cut
    # several workgroups per problem only where every workgroup gets a compute unit of the device to itself; this
    # process may have no device at all, and then the route asks for nothing
    gang = rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, 3, 8192, 256)
    assert gang == 0 or 0 < gang < one
    assert rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN, 1, 8192, 512) == 0
    # the segmented route for more problems
    assert rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SEGMENTED, 16, 8192, 256) == 16 * one
    assert rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SEGMENTED, 33, 8192, 256) == 0
    assert rh.rh_workspace_size(rh.WS_MINPLUS_CHAIN_SEGMENTED, 4, 127, 256) == 0
    pairs = 2 * 4097 * 16                      # two buffers of 16-byte pairs per problem
    assert rh.rh_workspace_size(rh.WS_STAGE_DP, 2, 4096, 64) >= 2 * pairs
    assert rh.rh_workspace_size(rh.WS_STAGE_DP, 64, 4096, 64) == 64 * pairs     # many problems: no split tiles
    assert rh.rh_workspace_size(rh.WS_STAGE_DP, 1, 10, 11) == 0                 # S > L is not a valid call
    # argument errors are found before anything touches a device
    L = rh.lib()
    assert L.rh_minplus_chain(1, 2, 100, None, 0, None, 0, None, None, None, None, None, 0, None) == -3
    assert L.rh_minplus_chain(1, 2, 128, None, 0, None, 0, None, None, None, None, None, 0, None) == -1
    assert L.rh_stage_dp(1, 10, 11, None, None, None, 0, None, None, 0, None) == -2
    assert L.rh_interval_costs(1, 8, 48, None, None, 10, None, None, 0, None) == -3
    assert L.rh_interval_costs(1, 8, 64, None, None, 9, None, None, 0, None) == -2      # odd row stride
    assert L.rh_stage_dp_interval(1, 8, 9, 10, None, None, None, 0, None, None, 0, None) == -2
    assert L.rh_interval_costs_banded(1, 8, 64, 0, None, None, 10, None, None, 0, None) == -2      # a stage holds an operator at least
    assert L.rh_stage_dp_interval_banded(1, 8, 4, 0, 10, None, None, None, 0, None, None, 0, None) == -2
    assert L.rh_stage_plans(1, 8, 64, 9, None, None, None, None, None, None, None, None) == -2      # more stages than operators
    assert L.rh_stage_plans(1, 8, 64, 2, None, None, None, None, None, None, None, None) == -1
    assert rh.rh_workspace_size(rh.WS_STAGE_DP_INTERVAL, 1, 4096, 64) > 2 * 4097 * 8
    # the table by blocks: Kp = 64 and at least four blocks of 128 operators
    assert rh.rh_workspace_size(rh.WS_INTERVAL_COSTS, 1, 4096, 64) > 32 * 32 * 64 * 64 * 8
    assert rh.rh_workspace_size(rh.WS_INTERVAL_COSTS, 1, 511, 64) == 0
    assert rh.rh_workspace_size(rh.WS_INTERVAL_COSTS, 1, 4096, 128) == 0
    assert L.rh_backtrack(-1, 2, 128, None, None, None, None) == -2
    assert L.rh_build_reshard(None, 1, 128, None, None, None, None, None, None, None) == -1
    assert L.rh_check_costs(None, 5, None, None) == -1


def test_workgroups_per_problem_follow_the_compute_units():
    # eight workgroups per problem while they all fit, then four, then the route is not taken
    g = rh.rh_gang_workgroups
    assert [g(B, 256) for B in (1, 32, 33, 64, 65)] == [8, 8, 4, 4, 0]
    assert [g(B, 304) for B in (38, 39, 76, 77)] == [8, 4, 4, 0]
    assert [g(B, 64) for B in (8, 9, 16, 17)] == [8, 4, 4, 0]
    assert g(1, 8) == 8 and g(1, 7) == 4 and g(1, 3) == 0 and g(1, 0) == 0      # a device with few units, or none
    assert g(0, 256) == 0 and g(-1, 256) == 0
    for cus in (1, 8, 60, 104, 256, 304):
        for B in range(1, 80):
            n = g(B, cus)
            assert n in (0, 4, 8) and B * n <= cus
            assert n == 8 or B * 8 > cus                                      # never fewer than what fits
