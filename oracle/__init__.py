"""ctypes loader of the CPU oracle (TEST INFRASTRUCTURE ONLY).

Only tests, the smoke check and the bench's CPU-baseline leg may import this
package.  It builds `oracle.c` with gcc on first use and exposes numpy-array
wrappers; it imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "oracle.c")
# ORACLE_SANITIZED=1 (set by the sanitizer test for a child process that preloads the AddressSanitizer runtime) loads a
# build with -fsanitize=address,undefined instead; the numbers are the same, every out-of-bounds access, overflow
# of a signed integer or misaligned pointer ends the process
SANITIZED = os.environ.get("ORACLE_SANITIZED") == "1"
_LIB = os.path.join(_HERE, "liboracle_san.so" if SANITIZED else "liboracle.so")
INF = 1 << 52

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc -O2 (no SIMD intrinsics, OpenMP across problems only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        flags = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer"] \
            if SANITIZED else ["-O2"]
        subprocess.check_call(["gcc"] + flags + ["-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
                                                 "-o", _LIB, _SRC])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.oracle_plan_cost.restype = ctypes.c_int64
        _lib.oracle_owner.restype = ctypes.c_int64
        _lib.oracle_owner.argtypes = [ctypes.c_int64] * 3
        _lib.oracle_axis_bytes.restype = ctypes.c_int64
    return _lib


def _p(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def _chk(a, dtype, name):
    if a.dtype != dtype or not a.flags["C_CONTIGUOUS"]:
        raise TypeError(f"{name}: need C-contiguous {dtype}")
    return a


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def chain(c: np.ndarray, R: np.ndarray, nthreads: int = 1, shared_R: bool = False):
    """c[B][N][Kp], R[B][N-1][Kp][Kp] (or [N-1][Kp][Kp] with shared_R) ->
    arg uint16[B][N-1][Kp], vfinal[B][Kp], total[B], last[B]."""
    _chk(c, np.int64, "c"); _chk(R, np.int64, "R")
    B, N, Kp = c.shape
    if shared_R:
        assert R.shape == (N - 1, Kp, Kp)
        r_bs = 0
    else:
        assert R.shape == (B, N - 1, Kp, Kp)
        r_bs = (N - 1) * Kp * Kp
    arg = np.zeros((B, max(N - 1, 0), Kp), dtype=np.uint16)
    vfinal = np.zeros((B, Kp), dtype=np.int64)
    total = np.zeros(B, dtype=np.int64)
    last = np.zeros(B, dtype=np.int32)
    rc = lib().oracle_chain(ctypes.c_int32(B), ctypes.c_int32(N), ctypes.c_int32(Kp), _p(c),
                            ctypes.c_int64(N * Kp), _p(R), ctypes.c_int64(r_bs), _p(arg),
                            _p(vfinal), _p(total), _p(last), ctypes.c_int32(nthreads))
    if rc != 0:
        raise ValueError(f"oracle_chain rc={rc}")
    return arg, vfinal, total, last


def backtrack(arg: np.ndarray, last: np.ndarray) -> np.ndarray:
    _chk(arg, np.uint16, "arg"); _chk(last, np.int32, "last")
    B, Nm1, Kp = arg.shape
    plan = np.zeros((B, Nm1 + 1), dtype=np.int32)
    rc = lib().oracle_backtrack(ctypes.c_int32(B), ctypes.c_int32(Nm1 + 1), ctypes.c_int32(Kp),
                                _p(arg), _p(last), _p(plan))
    if rc != 0:
        raise ValueError(f"oracle_backtrack rc={rc}")
    return plan


def plan_cost(c: np.ndarray, R: np.ndarray, plan: np.ndarray) -> int:
    """Objective of one plan on one problem: c[N][Kp], R[N-1][Kp][Kp], plan int32[N]."""
    _chk(c, np.int64, "c"); _chk(R, np.int64, "R"); _chk(plan, np.int32, "plan")
    N, Kp = c.shape
    return int(lib().oracle_plan_cost(ctypes.c_int32(N), ctypes.c_int32(Kp), _p(c), _p(R), _p(plan)))


def cone(branches, c_root: np.ndarray):
    """branches: list of (c[len][Kp], R[len][Kp][Kp]) with the last R the edge into the root; c_root[Kp] ->
    table[Kp], total, root_choice, [plan per branch]."""
    _chk(c_root, np.int64, "c_root")
    Kp = c_root.shape[0]
    n = len(branches)
    lens = np.array([b[0].shape[0] for b in branches], dtype=np.int32)
    for cb, Rb in branches:
        _chk(cb, np.int64, "branch c"); _chk(Rb, np.int64, "branch R")
        assert cb.shape[1] == Kp and Rb.shape == (cb.shape[0], Kp, Kp)
    PP = ctypes.c_void_p * max(n, 1)
    cps = PP(*[b[0].ctypes.data for b in branches])
    rps = PP(*[b[1].ctypes.data for b in branches])
    plans = [np.zeros(int(l), dtype=np.int32) for l in lens]
    pps = PP(*[p.ctypes.data for p in plans])
    table = np.zeros(Kp, dtype=np.int64)
    total = np.zeros(1, dtype=np.int64)
    choice = np.zeros(1, dtype=np.int32)
    rc = lib().oracle_cone(ctypes.c_int32(n), ctypes.c_int32(Kp), _p(lens), cps, rps, _p(c_root), _p(table),
                           _p(total), _p(choice), pps)
    if rc != 0:
        raise ValueError(f"oracle_cone rc={rc}")
    return table, int(total[0]), int(choice[0]), plans


def tree(parent: np.ndarray, c: np.ndarray, R: np.ndarray):
    """In-tree DP: parent int32[n] (parent[i] > i, root n-1 has -1), c[n][Kp], R[n-1][Kp][Kp] (edge i -> parent[i],
    row = strategy of i) -> table[Kp], total, root_choice, plan int32[n], arg uint16[n-1][Kp]."""
    _chk(parent, np.int32, "parent"); _chk(c, np.int64, "c"); _chk(R, np.int64, "R")
    n, Kp = c.shape
    assert parent.shape == (n,) and R.shape == (max(n - 1, 0), Kp, Kp)
    table = np.zeros(Kp, dtype=np.int64)
    total = np.zeros(1, dtype=np.int64)
    choice = np.zeros(1, dtype=np.int32)
    plan = np.zeros(n, dtype=np.int32)
    arg = np.zeros((max(n - 1, 0), Kp), dtype=np.uint16)
    rc = lib().oracle_tree(ctypes.c_int32(n), ctypes.c_int32(Kp), _p(parent), _p(c), _p(R), _p(table), _p(total),
                           _p(choice), _p(plan), _p(arg))
    if rc != 0:
        raise ValueError(f"oracle_tree rc={rc}")
    return table, int(total[0]), int(choice[0]), plan, arg


def memory_sweep(c, R, param_bytes, repl, mem, limit: int, n_k: int, k0: int = 0):
    """c[N][Kp], R[N-1][Kp][Kp], param_bytes int64[N], repl uint8[N][Kp], mem int64[N][Kp] ->
    total[n_k], plan int32[n_k][N], plan_mem[n_k], first (offset of the smallest feasible k, or -1)."""
    _chk(c, np.int64, "c"); _chk(R, np.int64, "R"); _chk(param_bytes, np.int64, "param_bytes")
    _chk(repl, np.uint8, "repl"); _chk(mem, np.int64, "mem")
    N, Kp = c.shape
    total = np.zeros(n_k, dtype=np.int64)
    plan = np.zeros((n_k, N), dtype=np.int32)
    plan_mem = np.zeros(n_k, dtype=np.int64)
    first = np.zeros(1, dtype=np.int32)
    rc = lib().oracle_memory_sweep(ctypes.c_int32(N), ctypes.c_int32(Kp), ctypes.c_int32(n_k), ctypes.c_int32(k0),
                                   _p(c), _p(R), _p(param_bytes), _p(repl), _p(mem), ctypes.c_int64(limit),
                                   _p(total), _p(plan), _p(plan_mem), _p(first))
    if rc != 0:
        raise ValueError(f"oracle_memory_sweep rc={rc}")
    return total, plan, plan_mem, int(first[0])


def stage_dp(cost: np.ndarray, S: int, s_query: int = 0, nthreads: int = 1):
    """cost[B][L] -> bottleneck[B][S], cut int32[B][S][L+1], bounds int32[B][s_query+1] or None."""
    _chk(cost, np.int64, "cost")
    B, L = cost.shape
    bott = np.zeros((B, S), dtype=np.int64)
    cut = np.zeros((B, S, L + 1), dtype=np.int32)
    bounds = np.zeros((B, s_query + 1), dtype=np.int32) if s_query > 0 else None
    rc = lib().oracle_stage_dp(ctypes.c_int32(B), ctypes.c_int32(L), ctypes.c_int32(S), _p(cost),
                               _p(bott), _p(cut), ctypes.c_int32(s_query),
                               _p(bounds) if bounds is not None else None,
                               ctypes.c_int32(nthreads))
    if rc != 0:
        raise ValueError(f"oracle_stage_dp rc={rc}")
    return bott, cut, bounds


def interval_costs(c: np.ndarray, R: np.ndarray, ldT: int = 0, nthreads: int = 1, max_len: int = 0) -> np.ndarray:
    """c[L][Kp], R[L-1][Kp][Kp] -> T int64[L][ldT] (ldT >= L+1, default L+1): T[i][j] = least plan cost of the
    operators i..j-1 on their own, INF where j <= i; columns beyond L are left at -1.  max_len > 0: no stage
    longer than max_len operators, T[i][j] = INF for j - i > max_len."""
    _chk(c, np.int64, "c"); _chk(R, np.int64, "R")
    L, Kp = c.shape
    assert R.shape == (max(L - 1, 0), Kp, Kp)
    ldT = ldT or L + 1
    T = np.full((L, ldT), -1, dtype=np.int64)
    if max_len > 0:
        rc = lib().oracle_interval_costs_banded(ctypes.c_int32(L), ctypes.c_int32(Kp), ctypes.c_int32(max_len),
                                                _p(c), _p(R), ctypes.c_int64(ldT), _p(T), ctypes.c_int32(nthreads))
    else:
        rc = lib().oracle_interval_costs(ctypes.c_int32(L), ctypes.c_int32(Kp), _p(c), _p(R), ctypes.c_int64(ldT),
                                         _p(T), ctypes.c_int32(nthreads))
    if rc != 0:
        raise ValueError(f"oracle_interval_costs rc={rc}")
    return T


def stage_interval(T: np.ndarray, S: int, s_query: int = 0, nthreads: int = 1):
    """T[B][L][ldT] -> bottleneck[B][S], cut int32[B][S][L+1], bounds int32[B][s_query+1] or None."""
    _chk(T, np.int64, "T")
    B, L, ldT = T.shape
    bott = np.zeros((B, S), dtype=np.int64)
    cut = np.zeros((B, S, L + 1), dtype=np.int32)
    bounds = np.zeros((B, s_query + 1), dtype=np.int32) if s_query > 0 else None
    rc = lib().oracle_stage_interval(ctypes.c_int32(B), ctypes.c_int32(L), ctypes.c_int32(S), ctypes.c_int64(ldT),
                                     _p(T), _p(bott), _p(cut), ctypes.c_int32(s_query),
                                     _p(bounds) if bounds is not None else None, ctypes.c_int32(nthreads))
    if rc != 0:
        raise ValueError(f"oracle_stage_interval rc={rc}")
    return bott, cut, bounds


def stage_window(cost: np.ndarray, d: int, xfer=None, eps_num: int = -1, eps_den: int = 1):
    """cost[B][L], xfer[B][L+1] or None -> bottleneck[B], cut int32[B][d][L+1], bounds int32[B][d+1]."""
    _chk(cost, np.int64, "cost")
    B, L = cost.shape
    if xfer is not None:
        _chk(xfer, np.int64, "xfer")
        assert xfer.shape == (B, L + 1)
    bott = np.zeros(B, dtype=np.int64)
    cut = np.zeros((B, d, L + 1), dtype=np.int32)
    bounds = np.zeros((B, d + 1), dtype=np.int32)
    rc = lib().oracle_stage_window(ctypes.c_int32(B), ctypes.c_int32(L), ctypes.c_int32(d), _p(cost),
                                   _p(xfer) if xfer is not None else None, ctypes.c_int64(eps_num),
                                   ctypes.c_int64(eps_den), _p(bott), _p(cut), _p(bounds))
    if rc != 0:
        raise ValueError(f"oracle_stage_window rc={rc}")
    return bott, cut, bounds


def build_reshard(m, bw_bytes_per_us, alpha_ns, K: np.ndarray, out_spec: np.ndarray,
                  in_spec: np.ndarray, dims: np.ndarray, elem_bytes: np.ndarray) -> np.ndarray:
    """Specs uint32[n_edges+1][Kp], dims int64[n_edges][4], elem_bytes int32[n_edges],
    K int32[n_edges+1] -> R int64[n_edges][Kp][Kp]."""
    _chk(K, np.int32, "K"); _chk(out_spec, np.uint32, "out_spec"); _chk(in_spec, np.uint32, "in_spec")
    _chk(dims, np.int64, "dims"); _chk(elem_bytes, np.int32, "elem_bytes")
    n_ops, Kp = out_spec.shape
    n_edges = n_ops - 1
    assert in_spec.shape == (n_ops, Kp) and K.shape == (n_ops,)
    assert dims.shape == (n_edges, 4) and elem_bytes.shape == (n_edges,)
    naxes = len(m)
    mm = np.array(list(m) + [1] * (2 - naxes), dtype=np.int32)
    bw = np.array(list(bw_bytes_per_us) + [1] * (2 - naxes), dtype=np.int64)
    al = np.array(list(alpha_ns) + [0] * (2 - naxes), dtype=np.int64)
    R = np.zeros((n_edges, Kp, Kp), dtype=np.int64)
    rc = lib().oracle_build_reshard(ctypes.c_int32(naxes), _p(mm), _p(bw), _p(al),
                                    ctypes.c_int32(n_edges), ctypes.c_int32(Kp), _p(K),
                                    _p(out_spec), _p(in_spec), _p(dims), _p(elem_bytes), _p(R))
    if rc != 0:
        raise ValueError(f"oracle_build_reshard rc={rc}")
    return R


def axis_bytes(p_byte: int, q_byte: int, dims, m: int, T: int) -> int:
    """Bytes one device receives on one mesh axis of size m for the transition p -> q
    of a local tensor of T bytes with extents dims[4]; -1 = impossible, -2 = invalid spec."""
    d = np.array(list(dims) + [1] * (4 - len(dims)), dtype=np.int64)
    return int(lib().oracle_axis_bytes(ctypes.c_uint32(p_byte), ctypes.c_uint32(q_byte), _p(d),
                                       ctypes.c_int32(m), ctypes.c_int64(T)))


def owner(u: int, stride: int, m: int) -> int:
    return int(lib().oracle_owner(u, stride, m))
