"""ctypes binding of librhino.so: same entry-point names, argument marshalling only.

Tensors are torch CUDA tensors (PyTorch is used for device memory and streams,
nothing else); every call is enqueued on torch's current stream.  There is no
CPU path: a missing library raises at first use.
"""
from __future__ import annotations

import ctypes
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
# RHINO_LIBRARY names another build of the same library (the CPU-side sanitizer leg of the tests uses it)
LIB_PATH = os.environ.get("RHINO_LIBRARY") or os.path.join(_PKG, "librhino.so")

INF = 1 << 52
KMIN, KMAX, NMAX = 16, 1024, 16384
WS_MINPLUS_CHAIN, WS_STAGE_DP, WS_STAGE_DP_WINDOW, WS_STAGE_DP_INTERVAL, WS_MINPLUS_CHAIN_SEGMENTED = 0, 1, 2, 3, 4
WS_MINPLUS_CHAIN_SPECS, WS_INTERVAL_COSTS = 5, 6


class RhinoError(RuntimeError):
    def __init__(self, code: int, what: str):
        super().__init__(f"{what}: {strerror(code)} (code {code})")
        self.code = code


class Mesh(ctypes.Structure):
    """Mirror of rh_mesh_t."""
    _fields_ = [("naxes", ctypes.c_int32), ("m", ctypes.c_int32 * 2),
                ("bw_bytes_per_us", ctypes.c_int64 * 2), ("alpha_ns", ctypes.c_int64 * 2)]

    @classmethod
    def make(cls, m, bw_bytes_per_us, alpha_ns=None):
        n = len(m)
        alpha_ns = [0] * n if alpha_ns is None else list(alpha_ns)
        pad = lambda xs, v: list(xs) + [v] * (2 - n)
        return cls(n, (ctypes.c_int32 * 2)(*pad(m, 1)), (ctypes.c_int64 * 2)(*pad(bw_bytes_per_us, 1)),
                   (ctypes.c_int64 * 2)(*pad(alpha_ns, 0)))


_lib = None


def lib():
    """Load the HIP library built in-tree; fail loudly if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2302_08141_amd.build` "
                               "(there is no CPU fallback)")
        L = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        L.rh_build_reshard.argtypes = [ctypes.POINTER(Mesh), i32, i32, vp, vp, vp, vp, vp, vp, vp]
        L.rh_minplus_chain.argtypes = [i32, i32, i32, vp, i64, vp, i64, vp, vp, vp, vp, vp, sz, vp]
        L.rh_minplus_chain_specs.argtypes = [i32, i32, i32, i32, ctypes.POINTER(Mesh), vp, i64, vp, vp, vp, vp, vp, vp, vp,
                                             vp, vp, vp, sz, vp]
        L.rh_minplus_chain_specs.restype = ctypes.c_int
        L.rh_backtrack.argtypes = [i32, i32, i32, vp, vp, vp, vp]
        L.rh_stage_dp.argtypes = [i32, i32, i32, vp, vp, vp, i32, vp, vp, sz, vp]
        L.rh_cone_merge.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.rh_cone_merge.restype = ctypes.c_int
        L.rh_tree_plan.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp]
        L.rh_tree_dp.argtypes = [i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, i64, vp, i64, vp, vp, vp, vp, vp, vp]
        L.rh_tree_plan.restype = L.rh_tree_dp.restype = ctypes.c_int
        L.rh_mask_replicated.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp]
        L.rh_plan_memory.argtypes = [i32, i32, i32, vp, vp, vp, i64, vp, vp, vp]
        L.rh_mask_replicated.restype = L.rh_plan_memory.restype = ctypes.c_int
        L.rh_stage_dp_window.argtypes = [i32, i32, i32, vp, vp, i64, i64, vp, vp, vp, vp, sz, vp]
        L.rh_stage_dp_window.restype = ctypes.c_int
        L.rh_stage_dp_window_static.argtypes = [i32, i32, i32, vp, vp, i64, i64, vp, vp, vp, vp]
        L.rh_stage_dp_window_static.restype = ctypes.c_int
        L.rh_static_scratch_bytes.argtypes = []
        L.rh_static_scratch_bytes.restype = sz
        L.rh_interval_costs.argtypes = [i32, i32, i32, vp, vp, i64, vp, vp, sz, vp]
        L.rh_stage_dp_interval.argtypes = [i32, i32, i32, i64, vp, vp, vp, i32, vp, vp, sz, vp]
        L.rh_stage_plans.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        L.rh_stage_plans.restype = ctypes.c_int
        L.rh_interval_costs_banded.argtypes = [i32, i32, i32, i32, vp, vp, i64, vp, vp, sz, vp]
        L.rh_stage_dp_interval_banded.argtypes = [i32, i32, i32, i32, i64, vp, vp, vp, i32, vp, vp, sz, vp]
        L.rh_interval_costs_banded.restype = L.rh_stage_dp_interval_banded.restype = ctypes.c_int
        L.rh_workspace_size.argtypes = [i32, i32, i32, i32]
        L.rh_workspace_size.restype = sz
        L.rh_check_costs.argtypes = [vp, i64, vp, vp]
        L.rh_gang_workgroups.argtypes = [i32, i32]
        L.rh_gang_workgroups.restype = ctypes.c_int
        L.rh_strerror.argtypes = [ctypes.c_int]
        L.rh_strerror.restype = ctypes.c_char_p
        for f in (L.rh_build_reshard, L.rh_minplus_chain, L.rh_backtrack, L.rh_stage_dp, L.rh_check_costs,
                  L.rh_version):
            f.restype = ctypes.c_int
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().rh_strerror(code).decode()


def rh_version() -> int:
    return lib().rh_version()


def rh_gang_workgroups(B: int, compute_units: int) -> int:
    return lib().rh_gang_workgroups(B, compute_units)


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t, dtype, name, need: int = 0):
    """Device pointer of t after checking type, layout and that it holds at least `need` elements
    (the kernels index by the sizes passed, so a short buffer must never reach them)."""
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.dtype == dtype and t.is_contiguous()):
        raise TypeError(f"{name}: need a contiguous CUDA tensor of {dtype}")
    if t.numel() < need:
        raise ValueError(f"{name}: {t.numel()} elements, the call needs {need}")
    return ctypes.c_void_p(t.data_ptr())


def _check(rc, what):
    if rc != 0:
        raise RhinoError(rc, what)


def rh_build_reshard(mesh: Mesh, n_edges: int, Kp: int, K, out_spec, in_spec, dims, elem_bytes, R):
    """K int32[n_edges+1]; out_spec, in_spec int32-typed words [n_edges+1][Kp]; dims int64[n_edges][4];
    elem_bytes int32[n_edges]; R int64[n_edges][Kp][Kp] (out)."""
    e, k = max(n_edges, 0), max(Kp, 0)
    _check(lib().rh_build_reshard(ctypes.byref(mesh), n_edges, Kp, _ptr(K, torch.int32, "K", e + 1),
                                  _ptr(out_spec, torch.int32, "out_spec", (e + 1) * k),
                                  _ptr(in_spec, torch.int32, "in_spec", (e + 1) * k),
                                  _ptr(dims, torch.int64, "dims", 4 * e),
                                  _ptr(elem_bytes, torch.int32, "elem_bytes", e),
                                  _ptr(R, torch.int64, "R", e * k * k), _stream()), "rh_build_reshard")


def rh_minplus_chain(B: int, N: int, Kp: int, c, c_batch_stride: int, R, R_batch_stride: int, arg, vfinal,
                     total, last, workspace=None):
    """c int64[B][N][Kp]; R int64[B][N-1][Kp][Kp] (or one shared table with R_batch_stride 0);
    arg: int16-typed storage for uint16[B][N-1][Kp] (out); vfinal int64[B][Kp] or None; total int64[B];
    last int32[B]; workspace: optional uint8 CUDA tensor of rh_workspace_size(WS_MINPLUS_CHAIN, B, N, Kp) bytes."""
    workspace_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    b, n, k = max(B, 0), max(N, 1), max(Kp, 0)
    span = lambda stride, one: (b - 1) * stride + one if b > 0 else 0     # elements the batch touches
    _check(lib().rh_minplus_chain(B, N, Kp, _ptr(c, torch.int64, "c", span(c_batch_stride, n * k)),
                                  c_batch_stride,
                                  _ptr(R, torch.int64, "R", span(R_batch_stride, (n - 1) * k * k)),
                                  R_batch_stride, _ptr(arg, torch.int16, "arg", b * (n - 1) * k),
                                  _ptr(vfinal, torch.int64, "vfinal", b * k), _ptr(total, torch.int64, "total", b),
                                  _ptr(last, torch.int32, "last", b),
                                  ctypes.c_void_p(workspace.data_ptr()) if workspace is not None else None,
                                  workspace_bytes, _stream()), "rh_minplus_chain")


def rh_minplus_chain_specs(B: int, N: int, Kp: int, meshes, c, c_batch_stride: int, K, out_spec, in_spec, dims,
                           elem_bytes, arg, vfinal, total, last, workspace=None):
    """meshes: list of at most 64 Mesh, problem p uses meshes[p % len(meshes)]; c int64[B][N][Kp]; K int32[N];
    out_spec, in_spec int32-typed words [N][Kp]; dims int64[N-1][4]; elem_bytes int32[N-1]; outputs as for
    rh_minplus_chain; workspace: optional uint8 tensor of rh_workspace_size(WS_MINPLUS_CHAIN_SPECS, B, N, Kp) bytes."""
    marr = (Mesh * max(len(meshes), 1))(*meshes)
    ws_ptr = ctypes.c_void_p(workspace.data_ptr()) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    b, n, k = max(B, 0), max(N, 1), max(Kp, 0)
    span = (b - 1) * c_batch_stride + n * k if b > 0 else 0
    _check(lib().rh_minplus_chain_specs(B, N, Kp, len(meshes), marr, _ptr(c, torch.int64, "c", span), c_batch_stride,
                                        _ptr(K, torch.int32, "K", n), _ptr(out_spec, torch.int32, "out_spec", n * k),
                                        _ptr(in_spec, torch.int32, "in_spec", n * k),
                                        _ptr(dims, torch.int64, "dims", 4 * (n - 1)),
                                        _ptr(elem_bytes, torch.int32, "elem_bytes", n - 1),
                                        _ptr(arg, torch.int16, "arg", b * (n - 1) * k),
                                        _ptr(vfinal, torch.int64, "vfinal", b * k), _ptr(total, torch.int64, "total", b),
                                        _ptr(last, torch.int32, "last", b), ws_ptr, ws_bytes, _stream()),
           "rh_minplus_chain_specs")


def rh_backtrack(B: int, N: int, Kp: int, arg, last, plan):
    b, n, k = max(B, 0), max(N, 1), max(Kp, 0)
    _check(lib().rh_backtrack(B, N, Kp, _ptr(arg, torch.int16, "arg", b * (n - 1) * k),
                              _ptr(last, torch.int32, "last", b), _ptr(plan, torch.int32, "plan", b * n),
                              _stream()), "rh_backtrack")


def rh_cone_merge(n_cones: int, n_branches: int, Kp: int, branch_start, w, c_root, table, total, root_choice,
                  branch_last):
    """branch_start int32[n_cones+1]; w int64[n_branches][Kp]; c_root int64[n_cones][Kp]; table int64[n_cones][Kp] or
    None; total int64[n_cones]; root_choice int32[n_cones]; branch_last int32[n_branches] or None."""
    q, b, k = max(n_cones, 0), max(n_branches, 0), max(Kp, 0)
    _check(lib().rh_cone_merge(n_cones, n_branches, Kp, _ptr(branch_start, torch.int32, "branch_start", q + 1),
                               _ptr(w, torch.int64, "w", b * k), _ptr(c_root, torch.int64, "c_root", q * k),
                               _ptr(table, torch.int64, "table", q * k), _ptr(total, torch.int64, "total", q),
                               _ptr(root_choice, torch.int32, "root_choice", q),
                               _ptr(branch_last, torch.int32, "branch_last", b), _stream()), "rh_cone_merge")


class TreePlan:
    """What rh_tree_plan returns for one parent array: the host arrays and device copies of those rh_tree_dp reads on
    the device."""

    def __init__(self, parent, device):
        import numpy as np
        parent = np.ascontiguousarray(parent, dtype=np.int32)
        n = parent.shape[0]
        self.n = n
        host = {k: np.zeros(n + 1, dtype=np.int32) for k in ("run_first", "run_last", "round_start", "child_start",
                                                              "child_list")}
        n_runs = ctypes.c_int32(0)
        hp = lambda a: a.ctypes.data_as(ctypes.c_void_p)
        rounds = lib().rh_tree_plan(n, hp(parent), hp(host["run_first"]), hp(host["run_last"]), hp(host["round_start"]),
                                    hp(host["child_start"]), hp(host["child_list"]), ctypes.byref(n_runs))
        _check(min(rounds, 0), "rh_tree_plan")
        self.n_rounds, self.n_runs = rounds, n_runs.value
        self.host = dict(host, parent=parent)
        self.round_start = host["round_start"]
        self.dev = {k: torch.from_numpy(v).to(device) for k, v in self.host.items() if k != "round_start"}


def rh_tree_dp(B: int, Kp: int, tp: TreePlan, c, c_batch_stride: int, R, R_batch_stride: int, arg, w, total,
               root_choice, plan):
    """tp: TreePlan; c int64[B][n][Kp]; R int64[B][n-1][Kp][Kp] (stride 0 = shared); arg int16[B][n-1][Kp];
    w int64[B][n][Kp]; total int64[B]; root_choice int32[B]; plan int32[B][n] or None."""
    n = tp.n
    b, k = max(B, 0), max(Kp, 0)
    c_span = (b - 1) * c_batch_stride + n * k if b > 0 else 0
    r_span = (b - 1) * R_batch_stride + (n - 1) * k * k if b > 0 else 0
    d = tp.dev
    _check(lib().rh_tree_dp(B, n, Kp, tp.n_runs, tp.n_rounds, tp.round_start.ctypes.data_as(ctypes.c_void_p),
                            _ptr(d["run_first"], torch.int32, "run_first", tp.n_runs),
                            _ptr(d["run_last"], torch.int32, "run_last", tp.n_runs),
                            _ptr(d["parent"], torch.int32, "parent", n),
                            _ptr(d["child_start"], torch.int32, "child_start", n + 1),
                            _ptr(d["child_list"], torch.int32, "child_list", n),
                            _ptr(c, torch.int64, "c", c_span), c_batch_stride, _ptr(R, torch.int64, "R", r_span),
                            R_batch_stride, _ptr(arg, torch.int16, "arg", b * (n - 1) * k),
                            _ptr(w, torch.int64, "w", b * n * k), _ptr(total, torch.int64, "total", b),
                            _ptr(root_choice, torch.int32, "root_choice", b), _ptr(plan, torch.int32, "plan", b * n),
                            _stream()), "rh_tree_dp")


def rh_mask_replicated(N: int, Kp: int, n_k: int, k0: int, c, param_bytes, repl, c_out):
    """c int64[N][Kp]; param_bytes int64[N]; repl uint8[N][Kp]; c_out int64[n_k][N][Kp] (out)."""
    n, k, t = max(N, 0), max(Kp, 0), max(n_k, 0)
    _check(lib().rh_mask_replicated(N, Kp, n_k, k0, _ptr(c, torch.int64, "c", n * k),
                                    _ptr(param_bytes, torch.int64, "param_bytes", n),
                                    _ptr(repl, torch.uint8, "repl", n * k),
                                    _ptr(c_out, torch.int64, "c_out", t * n * k), _stream()), "rh_mask_replicated")


def rh_plan_memory(B: int, N: int, Kp: int, plan, mem, total, limit: int, plan_mem, first):
    """plan int32[B][N]; mem int64[N][Kp]; total int64[B]; plan_mem int64[B] (out); first int32[1] (out) or None."""
    b, n, k = max(B, 0), max(N, 0), max(Kp, 0)
    _check(lib().rh_plan_memory(B, N, Kp, _ptr(plan, torch.int32, "plan", b * n), _ptr(mem, torch.int64, "mem", n * k),
                                _ptr(total, torch.int64, "total", b), limit,
                                _ptr(plan_mem, torch.int64, "plan_mem", b), _ptr(first, torch.int32, "first", 1),
                                _stream()), "rh_plan_memory")


def rh_workspace_size(which: int, B: int, N_or_L: int, Kp_or_S: int) -> int:
    return int(lib().rh_workspace_size(which, B, N_or_L, Kp_or_S))


def rh_stage_dp(B: int, L: int, S: int, seg_cost, bottleneck, cut, s_query: int, bounds, workspace):
    """seg_cost int64[B][L]; bottleneck int64[B][S]; cut int32[B][S][L+1]; bounds int32[B][s_query+1] or None;
    workspace: uint8 CUDA tensor of at least rh_workspace_size(WS_STAGE_DP, B, L, S) bytes."""
    ws_ptr = ctypes.c_void_p(workspace.data_ptr()) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    b, l, s_ = max(B, 0), max(L, 0), max(S, 0)
    _check(lib().rh_stage_dp(B, L, S, _ptr(seg_cost, torch.int64, "seg_cost", b * l),
                             _ptr(bottleneck, torch.int64, "bottleneck", b * s_),
                             _ptr(cut, torch.int32, "cut", b * s_ * (l + 1)), s_query,
                             _ptr(bounds, torch.int32, "bounds", b * (max(s_query, 0) + 1)), ws_ptr, ws_bytes,
                             _stream()), "rh_stage_dp")


def rh_stage_dp_window(B: int, L: int, S: int, seg_cost, xfer, eps_num: int, eps_den: int, bottleneck, cut, bounds,
                       workspace):
    """seg_cost int64[B][L]; xfer int64[B][L+1] or None; bottleneck int64[B]; cut int32[B][S][L+1];
    bounds int32[B][S+1] or None; workspace: uint8 tensor of rh_workspace_size(WS_STAGE_DP_WINDOW, B, L, S) bytes."""
    ws_ptr = ctypes.c_void_p(workspace.data_ptr()) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    b, l, s_ = max(B, 0), max(L, 0), max(S, 0)
    _check(lib().rh_stage_dp_window(B, L, S, _ptr(seg_cost, torch.int64, "seg_cost", b * l),
                                    _ptr(xfer, torch.int64, "xfer", b * (l + 1)), eps_num, eps_den,
                                    _ptr(bottleneck, torch.int64, "bottleneck", b),
                                    _ptr(cut, torch.int32, "cut", b * s_ * (l + 1)),
                                    _ptr(bounds, torch.int32, "bounds", b * (s_ + 1)), ws_ptr, ws_bytes, _stream()),
           "rh_stage_dp_window")


def rh_stage_dp_window_static(B: int, L: int, S: int, seg_cost, xfer, eps_num: int, eps_den: int, bottleneck, cut,
                              bounds):
    """rh_stage_dp_window on the library's own static scratch (no workspace, nothing allocated)."""
    b, l, s_ = max(B, 0), max(L, 0), max(S, 0)
    _check(lib().rh_stage_dp_window_static(B, L, S, _ptr(seg_cost, torch.int64, "seg_cost", b * l),
                                           _ptr(xfer, torch.int64, "xfer", b * (l + 1)), eps_num, eps_den,
                                           _ptr(bottleneck, torch.int64, "bottleneck", b),
                                           _ptr(cut, torch.int32, "cut", b * s_ * (l + 1)),
                                           _ptr(bounds, torch.int32, "bounds", b * (s_ + 1)), _stream()),
           "rh_stage_dp_window_static")


def rh_static_scratch_bytes() -> int:
    return int(lib().rh_static_scratch_bytes())


def rh_interval_costs(B: int, L: int, Kp: int, c, R, ldT: int, T, workspace=None):
    """c int64[B][L][Kp]; R int64[B][L-1][Kp][Kp] (None if L == 1); T int64[B][L][ldT] out, ldT even and > L;
    workspace: optional uint8 tensor of rh_workspace_size(WS_INTERVAL_COSTS, B, L, Kp) bytes."""
    b, l, k = max(B, 0), max(L, 0), max(Kp, 0)
    ws_ptr = ctypes.c_void_p(workspace.data_ptr()) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().rh_interval_costs(B, L, Kp, _ptr(c, torch.int64, "c", b * l * k),
                                   _ptr(R, torch.int64, "R", b * max(l - 1, 0) * k * k), ldT,
                                   _ptr(T, torch.int64, "T", b * l * max(ldT, 0)), ws_ptr, ws_bytes, _stream()),
           "rh_interval_costs")


def rh_stage_dp_interval(B: int, L: int, S: int, ldT: int, T, bottleneck, cut, s_query: int, bounds, workspace):
    """T int64[B][L][ldT]; bottleneck int64[B][S]; cut int32[B][S][L+1]; bounds int32[B][s_query+1] or None;
    workspace: uint8 tensor of rh_workspace_size(WS_STAGE_DP_INTERVAL, B, L, S) bytes."""
    ws_ptr = ctypes.c_void_p(workspace.data_ptr()) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    b, l, s_ = max(B, 0), max(L, 0), max(S, 0)
    _check(lib().rh_stage_dp_interval(B, L, S, ldT, _ptr(T, torch.int64, "T", b * l * max(ldT, 0)),
                                      _ptr(bottleneck, torch.int64, "bottleneck", b * s_),
                                      _ptr(cut, torch.int32, "cut", b * s_ * (l + 1)), s_query,
                                      _ptr(bounds, torch.int32, "bounds", b * (max(s_query, 0) + 1)), ws_ptr,
                                      ws_bytes, _stream()), "rh_stage_dp_interval")


def rh_interval_costs_banded(B: int, L: int, Kp: int, max_len: int, c, R, ldT: int, T, workspace=None):
    """rh_interval_costs with no stage longer than max_len operators: T[i][j] = RH_INF for j - i > max_len.
    workspace: optional uint8 tensor of rh_workspace_size(WS_INTERVAL_COSTS, B, L, Kp) bytes."""
    b, l, k = max(B, 0), max(L, 0), max(Kp, 0)
    ws_ptr = ctypes.c_void_p(workspace.data_ptr()) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().rh_interval_costs_banded(B, L, Kp, max_len, _ptr(c, torch.int64, "c", b * l * k),
                                          _ptr(R, torch.int64, "R", b * max(l - 1, 0) * k * k), ldT,
                                          _ptr(T, torch.int64, "T", b * l * max(ldT, 0)), ws_ptr, ws_bytes, _stream()),
           "rh_interval_costs_banded")


def rh_stage_plans(B: int, L: int, Kp: int, S: int, bounds, c, R, arg, stage_total, stage_last, plan):
    """bounds int32[B][S+1]; c int64[B][L][Kp]; R int64[B][L-1][Kp][Kp] (None if L == 1); arg int16[B][L-1][Kp] out;
    stage_total int64[B][S] out; stage_last int32[B][S] out; plan int32[B][L] out or None."""
    b, l, k, s_ = max(B, 0), max(L, 0), max(Kp, 0), max(S, 0)
    _check(lib().rh_stage_plans(B, L, Kp, S, _ptr(bounds, torch.int32, "bounds", b * (s_ + 1)),
                                _ptr(c, torch.int64, "c", b * l * k),
                                _ptr(R, torch.int64, "R", b * max(l - 1, 0) * k * k),
                                _ptr(arg, torch.int16, "arg", b * max(l - 1, 0) * k),
                                _ptr(stage_total, torch.int64, "stage_total", b * s_),
                                _ptr(stage_last, torch.int32, "stage_last", b * s_),
                                _ptr(plan, torch.int32, "plan", b * l), _stream()), "rh_stage_plans")


def rh_stage_dp_interval_banded(B: int, L: int, S: int, max_len: int, ldT: int, T, bottleneck, cut, s_query: int,
                                bounds, workspace):
    """rh_stage_dp_interval over stages of at most max_len operators (same buffers and workspace)."""
    ws_ptr = ctypes.c_void_p(workspace.data_ptr()) if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    b, l, s_ = max(B, 0), max(L, 0), max(S, 0)
    _check(lib().rh_stage_dp_interval_banded(B, L, S, max_len, ldT, _ptr(T, torch.int64, "T", b * l * max(ldT, 0)),
                                             _ptr(bottleneck, torch.int64, "bottleneck", b * s_),
                                             _ptr(cut, torch.int32, "cut", b * s_ * (l + 1)), s_query,
                                             _ptr(bounds, torch.int32, "bounds", b * (max(s_query, 0) + 1)), ws_ptr,
                                             ws_bytes, _stream()), "rh_stage_dp_interval_banded")


def rh_check_costs(x, violations):
    """Adds to violations (int64[1], caller-zeroed) the number of entries of x outside the cost contract."""
    _check(lib().rh_check_costs(_ptr(x, torch.int64, "x"), x.numel(), _ptr(violations, torch.int64, "violations"),
                                _stream()), "rh_check_costs")
