"""Transformer-shaped operator chains as search inputs (host side, numpy).

Stand-ins for the GPT and GShard-MoE graphs the paper evaluates on (Sec. 7.1,
Tables 1-2), linearised into a chain of operators as the segment-level search
of Sec. 4.3.2 sees it.  For every operator and every candidate strategy this
module emits what plan scoring takes as INPUT: the sharding spec of the
operator's output (`out_spec`), the spec it needs on its input (`in_spec`),
and its node cost c (compute time + local memory time in integer ns).  The
edge costs are NOT computed here -- that is the reshard builder's job.

A strategy slot is a pair (option on mesh axis 0, option on mesh axis 1) for
the operator's OUTPUT tensor; an option is replicate, partial, or split of one
tensor dim with stride = maximum >> lgdiv (Sec. 4.1, Sec. 4.3.3).  What the
operator then needs on its input follows from the operator kind:
  elementwise   same layout in and out (partial passes only through linear ops)
  matmul        batch/row dims carry over; a split output column dim needs a
                replicated input; a partial output comes from splitting the
                contracted (last) input dim
A slot whose specs are not valid layouts of the tensors involved stays in the
table with c = INF, so tables keep a uniform width.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from . import specs as sp
from .synthetic import INF

COST_CAP = (1 << 36) - 1      # finite costs stay inside the cost contract


@dataclass
class Op:
    name: str
    in_dims: tuple            # extents of the input tensor (rank <= 4)
    out_dims: tuple           # extents of the output tensor
    dim_map: dict             # output dim -> input dim carrying the same split, or None = input replicated
    partial_in: object        # None: partial output impossible; "P": passes through; (dim, lgdiv): split input dim
    flops: int
    bytes: int                # bytes the operator touches when not sharded (inputs + outputs + weights)
    weight_bytes: int = 0     # size of the operator's parameter tensor (0: none)


def elementwise(name, dims, eb, linear=False, n_inputs=1):
    n = int(np.prod(dims))
    return Op(name, dims, dims, {d: d for d in range(len(dims))}, "P" if linear else None, 2 * n * n_inputs,
              (n_inputs + 1) * n * eb)


def matmul(name, in_dims, out_dims, eb, k, n, dim_map=None, partial_in=None):
    """Rows = all dims but the last; contracts the last input dim (k) into n output columns."""
    rows = int(np.prod(out_dims)) // out_dims[-1] if dim_map is None else int(np.prod(out_dims)) // n
    last_in, last_out = len(in_dims) - 1, len(out_dims) - 1
    if dim_map is None:
        dim_map = {d: d for d in range(last_out)}
        dim_map[last_out] = None
    if partial_in is None:
        partial_in = (last_in, 0)
    return Op(name, in_dims, out_dims, dim_map, partial_in, 2 * rows * k * n,
              (int(np.prod(in_dims)) + int(np.prod(out_dims)) + k * n) * eb, weight_bytes=k * n * eb)


def pad4(dims):
    return tuple(dims) + (1,) * (4 - len(dims))


def spec_ok(word, dims, mesh):
    """Is the word a valid layout of a tensor with these extents on this mesh?"""
    axes = sp.unpack(word)[: len(mesh)]
    for x, (state, d, lg) in enumerate(axes):
        if state == 3:
            return False
        if state == sp.SPLIT and (d >= len(dims) or dims[d] % (mesh[x] << lg) != 0):
            return False
    if len(mesh) == 2 and axes[0][0] == sp.SPLIT and axes[1][0] == sp.SPLIT and axes[0][1] == axes[1][1]:
        return False
    return True


def options(rank, lgs, extra=()):
    """Per-axis options: replicate, partial, every dim at every listed stride, plus extras (dim, lgdiv)."""
    return [("R",), ("P",)] + [("S", d, lg) for d in range(rank) for lg in lgs] + [("S", d, lg) for d, lg in extra]


def _byte(opt):
    return sp.R_ if opt[0] == "R" else sp.P_ if opt[0] == "P" else sp.S_(opt[1], opt[2])


def _input_option(op: Op, opt):
    """Option needed on the input for this output option on one axis; None = impossible."""
    if opt[0] == "R":
        return ("R",)
    if opt[0] == "P":
        if op.partial_in is None:
            return None
        return ("P",) if op.partial_in == "P" else ("S", op.partial_in[0], op.partial_in[1])
    d_in = op.dim_map.get(opt[1], None)
    return ("R",) if d_in is None else ("S", d_in, opt[2])


def _shards_weight(op: Op, opt) -> bool:
    """Does this output option split the operator's parameter tensor along the axis?  A split output dim that
    the input does not carry is a parameter dim (column split); a partial output comes from splitting the
    contracted dim of input and parameter (row split)."""
    if opt[0] == "P":
        return isinstance(op.partial_in, tuple)
    return opt[0] == "S" and op.dim_map.get(opt[1], None) is None


def build_chain(ops, opts, mesh, peak_flop_per_ns, hbm_bytes_per_ns, Kp, eb):
    """-> dict with K, out_spec, in_spec (uint32[N][Kp]), dims (int64[N-1][4]), elem_bytes, c (int64[N][Kp]),
    and for the memory-constrained search param_bytes (int64[N]), repl (uint8[N][Kp]: the strategy keeps a full
    copy of the parameter), mem (int64[N][Kp]: parameter bytes per device)."""
    N, no = len(ops), len(opts)
    assert no * no <= Kp
    out_spec = np.full((N, Kp), sp.EMPTY, dtype=np.uint32)
    in_spec = np.full((N, Kp), sp.EMPTY, dtype=np.uint32)
    c = np.full((N, Kp), INF, dtype=np.int64)
    repl = np.zeros((N, Kp), dtype=np.uint8)
    mem = np.zeros((N, Kp), dtype=np.int64)
    param_bytes = np.array([op.weight_bytes for op in ops], dtype=np.int64)
    cache = {}
    for i, op in enumerate(ops):
        key = (op.in_dims, op.out_dims, tuple(sorted(op.dim_map.items(), key=str)), str(op.partial_in), op.flops,
               op.bytes, op.weight_bytes)
        if key not in cache:
            o_row = np.full(Kp, sp.EMPTY, dtype=np.uint32)
            i_row = np.full(Kp, sp.EMPTY, dtype=np.uint32)
            c_row = np.full(Kp, INF, dtype=np.int64)
            r_row = np.zeros(Kp, dtype=np.uint8)
            m_row = np.zeros(Kp, dtype=np.int64)
            for j0, a0 in enumerate(opts):
                for j1, a1 in enumerate(opts):
                    j = j0 * no + j1
                    ow = sp.word(_byte(a0), _byte(a1))
                    o_row[j] = ow
                    wshards = 1
                    for x, a in enumerate((a0, a1)):
                        if _shards_weight(op, a):
                            wshards *= mesh[x]
                    r_row[j] = 1 if (op.weight_bytes > 0 and wshards == 1) else 0
                    m_row[j] = op.weight_bytes // wshards
                    b0, b1 = _input_option(op, a0), _input_option(op, a1)
                    if b0 is None or b1 is None:
                        continue                      # in_spec stays EMPTY: the operator cannot do this
                    iw = sp.word(_byte(b0), _byte(b1))
                    i_row[j] = iw
                    if not (spec_ok(ow, op.out_dims, mesh) and spec_ok(iw, op.in_dims, mesh)):
                        continue
                    shards = 1
                    for x, a in enumerate((a0, a1)):
                        if a[0] != "R":
                            shards *= mesh[x]
                    cost = op.flops // shards // peak_flop_per_ns + op.bytes // shards // hbm_bytes_per_ns
                    c_row[j] = min(cost, COST_CAP)
            cache[key] = (o_row, i_row, c_row, r_row, m_row)
        out_spec[i], in_spec[i], c[i], repl[i], mem[i] = cache[key]
    for i in range(N - 1):
        assert pad4(ops[i].out_dims) == pad4(ops[i + 1].in_dims), (ops[i].name, ops[i + 1].name)
    dims = np.array([pad4(op.out_dims) for op in ops[:-1]], dtype=np.int64).reshape(N - 1, 4)
    return dict(N=N, Kp=Kp, K=np.full(N, no * no, dtype=np.int32), out_spec=out_spec, in_spec=in_spec, dims=dims,
                elem_bytes=np.full(N - 1, eb, dtype=np.int32), c=c, names=[op.name for op in ops], mesh=tuple(mesh),
                param_bytes=param_bytes, repl=repl, mem=mem)


# ---------------------------------------------------------------------------------------------
# GPT-like chain: 24 layers x 10 operators + embedding + head; hidden 4096, seq 2048, batch 8, fp16;
# logical 8x8 mesh; 8 options per axis -> K = 64.

GPT_MESH = dict(m=(8, 8), bw_bytes_per_us=(12_500, 150_000), alpha_ns=(0, 0))   # 100 Gb/s inter-node, fast intra-node
GPT_PEAK_FLOP_PER_NS = 1_000_000       # 1 PFLOP/s fp16
GPT_HBM_BYTES_PER_NS = 8_000           # 8 TB/s


def gpt_layer_ops(b, s, h, nh, eb):
    act, qkv, sc, ff = (b, s, h), (b, s, 3 * h), (b * nh, s, s), (b, s, 4 * h)
    hd = h // nh
    return [
        elementwise("ln1", act, eb),
        matmul("qkv", act, qkv, eb, h, 3 * h),
        # scores[b*nh, s, s]: batch*heads follows the batch dim of qkv, both seq dims follow its seq dim;
        # a partial result comes from splitting the head dim (half stride of the packed hidden dim)
        Op("score", qkv, sc, {0: 0, 1: 1, 2: 1}, (2, 1), 2 * b * nh * s * s * hd, (b * s * 3 * h + b * nh * s * s) * eb),
        # context[b, s, h]: contracts the key dim of the scores
        Op("av", sc, act, {0: 0, 1: 1, 2: None}, (2, 0), 2 * b * nh * s * s * hd, (b * nh * s * s + 2 * b * s * h) * eb),
        matmul("proj", act, act, eb, h, h),
        elementwise("add1", act, eb, linear=True, n_inputs=2),
        elementwise("ln2", act, eb),
        matmul("fc1", act, ff, eb, h, 4 * h),
        matmul("fc2", ff, act, eb, 4 * h, h),
        elementwise("add2", act, eb, linear=True, n_inputs=2),
    ]


def gpt_chain(layers=24, b=8, s=2048, h=4096, nh=32, vocab=32768, eb=2, Kp=64, m=None):
    """m: another logical mesh shape for the same graph (mesh shapes are enumerated by the search, Sec. 3)."""
    mesh = dict(GPT_MESH, m=tuple(m) if m is not None else GPT_MESH["m"])
    act = (b, s, h)
    ops = [elementwise("embed", act, eb, linear=True)]
    for _ in range(layers):
        ops += gpt_layer_ops(b, s, h, nh, eb)
    ops.append(matmul("head", act, (b, s, vocab), eb, h, vocab))
    g = build_chain(ops, options(3, (0, 1)), mesh["m"], GPT_PEAK_FLOP_PER_NS, GPT_HBM_BYTES_PER_NS, Kp, eb)
    g.update(mesh)
    return g


# ---------------------------------------------------------------------------------------------
# MoE-transformer-shaped chain: 96 layers x 85 operators + 32 = 8192 operators; hidden 12288, 64 experts,
# rank-4 tensors; logical 32x32 mesh; 16 options per axis -> K = 256.

MOE_MESH = dict(m=(32, 32), bw_bytes_per_us=(50_000, 400_000), alpha_ns=(0, 0))  # 400 Gb/s NIC, fast intra-node
MOE_PEAK_FLOP_PER_NS = 2_500_000       # 2.5 PFLOP/s
MOE_HBM_BYTES_PER_NS = 8_000


def moe_layer_ops(b, s, h, nh, E, eb):
    hd = h // nh
    act = (b, s, h, 1)                     # activations, hidden on dim 2
    heads = (b, s, nh, hd)                 # per-head view
    qkv = (b, s, 3 * nh, hd)
    sc = (b, nh, s, s)
    C = 2 * s // E                         # capacity per expert and group (top-2 routing)
    disp = (b, E, C, h)                    # dispatched tokens [G, E, C, H]
    eff = (b, E, C, 4 * h)
    gate = (b, s, E, 1)
    n_act = b * s * h

    def aux(name, dims, linear=True):
        return elementwise(name, dims, eb, linear=linear)

    fwd = [
        aux("ln1", act, linear=False),
        Op("qkv", act, qkv, {0: 0, 1: 1, 2: None, 3: None}, (2, 0), 2 * b * s * h * 3 * h, (4 * n_act + 3 * h * h) * eb,
           weight_bytes=3 * h * h * eb),
        aux("qkv_bias", qkv),
        Op("score", qkv, sc, {0: 0, 1: 2, 2: 1, 3: 1}, (3, 0), 2 * b * nh * s * s * hd, (3 * n_act + b * nh * s * s) * eb),
        aux("softmax", sc, linear=False),
        aux("attn_dropout", sc),
        Op("av", sc, heads, {0: 0, 1: 3, 2: 1, 3: None}, (3, 0), 2 * b * nh * s * s * hd, (b * nh * s * s + 2 * n_act) * eb),
        aux("merge_heads", heads),
        Op("proj", heads, act, {0: 0, 1: 1, 2: None, 3: None}, (2, 0), 2 * b * s * h * h, (2 * n_act + h * h) * eb,
           weight_bytes=h * h * eb),
        aux("proj_bias", act),
        elementwise("add1", act, eb, linear=True, n_inputs=2),
        aux("ln2", act, linear=False),
        Op("gate", act, gate, {0: 0, 1: 1, 2: None, 3: None}, (2, 0), 2 * b * s * h * E, (n_act + b * s * E + h * E) * eb,
           weight_bytes=h * E * eb),
        aux("gate_softmax", gate, linear=False),
        # routing: the gate scores choose where tokens go; as a chain operator it turns [b, s, E] into [G, E, C, H]
        Op("dispatch", gate, disp, {0: 0, 1: 2, 2: None, 3: None}, None, 2 * b * E * C * h, (n_act + b * E * C * h) * eb),
        aux("dispatch_cast", disp),
        Op("expert_fc1", disp, eff, {0: 0, 1: 1, 2: 2, 3: None}, (3, 0), 2 * b * E * C * h * 4 * h,
           (5 * b * E * C * h + E * 4 * h * h) * eb, weight_bytes=E * 4 * h * h * eb),
        aux("expert_bias1", eff),
        aux("expert_act", eff, linear=False),
        Op("expert_fc2", eff, disp, {0: 0, 1: 1, 2: 2, 3: None}, (3, 0), 2 * b * E * C * h * 4 * h,
           (5 * b * E * C * h + E * 4 * h * h) * eb, weight_bytes=E * 4 * h * h * eb),
        aux("expert_bias2", disp),
        Op("combine", disp, act, {0: 0, 1: None, 2: 3, 3: None}, (1, 0), 2 * b * E * C * h, (n_act + b * E * C * h) * eb),
        aux("combine_cast", act),
        elementwise("add2", act, eb, linear=True, n_inputs=2),
        aux("residual_dropout", act),
    ]
    return fwd


def _backward_of(op: Op, eb) -> Op:
    """The gradient twin: shapes swapped, the same flops again (dX), layouts follow the inverse dim map."""
    inv = {}
    for d_out, d_in in op.dim_map.items():
        if d_in is not None and d_in not in inv:
            inv[d_in] = d_out
    dim_map = {d: inv.get(d, None) for d in range(len(op.in_dims))}
    lin = op.partial_in == "P"
    # a replicated forward input dim that was split on the output side makes the gradient partial there
    split_only_out = [d for d, di in op.dim_map.items() if di is None]
    partial_in = "P" if lin else ((split_only_out[0], 0) if split_only_out else None)
    return Op("d_" + op.name, op.out_dims, op.in_dims, dim_map, partial_in, op.flops, op.bytes)


def moe_chain(layers=96, b=32, s=1024, h=12288, nh=96, E=64, eb=2, Kp=256, per_layer=85, tail=32):
    act = (b, s, h, 1)
    fwd = moe_layer_ops(b, s, h, nh, E, eb)
    bwd = [_backward_of(op, eb) for op in reversed(fwd)]
    layer = fwd + bwd
    # bookkeeping operators of the lowered graph (casts, gradient accumulation, optimizer slices) on the activation
    k = 0
    while len(layer) < per_layer:
        layer.append(elementwise(f"grad_accum{k}", act, eb, linear=True))
        k += 1
    assert len(layer) == per_layer, len(layer)
    ops = []
    for _ in range(layers):
        ops += layer
    ops += [elementwise(f"tail{t}", act, eb, linear=(t % 2 == 0)) for t in range(tail)]
    opts = options(4, (0, 1, 2), extra=((2, 3), (2, 4)))
    g = build_chain(ops, opts, MOE_MESH["m"], MOE_PEAK_FLOP_PER_NS, MOE_HBM_BYTES_PER_NS, Kp, eb)
    g.update(MOE_MESH)
    return g
