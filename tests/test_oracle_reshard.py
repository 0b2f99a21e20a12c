"""Pins of the resharding-cost oracle (CPU only).

The paper names the collectives (Sec. 2.1) and defines the specs (Sec. 4.1,
Sec. 4.3.3) but prints no volumes; the oracle counts units.  It is pinned by
the worked count of Sec. 4.3.3, hand-worked collective volumes, element-level
ownership on a tiny tensor, and the invariants the paper states (matched specs
need no communication, Sec. 4.1; uniform strides change nothing, Sec. 4.3.3).
"""
import itertools
import os

import numpy as np
import pytest

import oracle
from paper_2302_08141_amd.workloads import specs as sp

INF = oracle.INF


def _rows(path):
    with open(path) as f:
        return [ln.split() for ln in f if ln.strip() and not ln.startswith("#")]


def test_sharding_method_count_of_the_paper(golden_dir):
    n0, n1, ndev, methods, per_dim = map(int, _rows(os.path.join(golden_dir, "sharding_count.txt"))[0])
    dims = (n0, n1)
    count = 2                                               # replicate, partial
    for d, n in enumerate(dims):
        regular = 0
        for st in range(1, n // ndev + 1):                  # maximum stride = extent / shards
            owned = np.bincount([oracle.owner(u, st, ndev) for u in range(n)], minlength=ndev)
            regular += int(np.all(owned == n // ndev))      # every device holds an equal share
        assert regular == per_dim
        count += regular
        # the 3-bit lgdiv field reaches exactly these strides
        valid = [lg for lg in range(8) if oracle.axis_bytes(sp.S_(d, lg), sp.R_, dims, ndev, n0 * n1) != -2]
        assert valid == list(range(per_dim))
    assert count == methods


def test_owner_is_block_cyclic():
    # stride = consecutive units per block: 4 units, 2 shards
    assert [oracle.owner(u, 2, 2) for u in range(4)] == [0, 0, 1, 1]      # maximum stride
    assert [oracle.owner(u, 1, 2) for u in range(4)] == [0, 1, 0, 1]      # stride 1
    assert [oracle.owner(u, 2, 4) for u in range(16)] == [0, 0, 1, 1, 2, 2, 3, 3] * 2


def test_hand_worked_volumes(golden_dir):
    dims = (8, 2048, 4096)
    kinds = {
        "all_gather": (sp.S_(1), sp.R_),
        "reduce_scatter": (sp.P_, sp.S_(2)),
        "all_reduce": (sp.P_, sp.R_),
        "all_to_all_dim": (sp.S_(0), sp.S_(2)),
        "all_to_all_str": (sp.S_(2, 0), sp.S_(2, 1)),
    }
    for kind, local, m, nbytes, ns_slow, ns_fast in _rows(os.path.join(golden_dir, "reshard_volumes.txt")):
        local, m, nbytes, ns_slow, ns_fast = map(int, (local, m, nbytes, ns_slow, ns_fast))
        p, q = kinds[kind]
        assert oracle.axis_bytes(p, q, dims, m, local) == nbytes, kind
        # and through the full builder: the axis under test is axis 0; axis 1 either
        # replicates (local = whole tensor) or splits dim 0 / stays split (local = 1/8)
        other = sp.R_ if local == 134217728 else sp.S_(0)
        if other != sp.R_ and kind == "all_to_all_dim":
            p, q = sp.S_(1), sp.S_(2)                       # dim 0 is taken by axis 1
        for bw, want in ((12500, ns_slow), (150000, ns_fast)):
            R = oracle.build_reshard(
                (m, 8), (bw, 1), (0, 0), np.array([1, 1], np.int32),
                np.array([[sp.word(p, other)], [0]], np.uint32), np.array([[0], [sp.word(q, other)]], np.uint32),
                np.array([[8, 2048, 4096, 1]], np.int64), np.array([2], np.int32))
            assert R[0, 0, 0] == want, (kind, bw)


def _all_specs(ndims, lgs=(0, 1)):
    opts = [sp.R_, sp.P_] + [sp.S_(d, lg) for d in range(ndims) for lg in lgs]
    return [sp.word(a, b) for a in opts for b in opts]


def _owned(spec_axes, dims, mesh, dev):
    """Boolean tensor: which elements device `dev` holds under per-axis (state, dim, stride)."""
    own = np.ones(dims, dtype=bool)
    for x, (state, d, stride) in enumerate(spec_axes):
        if state != sp.SPLIT:
            continue
        # Sec. 4.1: blocks of `stride` consecutive units are dealt to the shards in turn (written out here, not
        # taken from the oracle; test_owner_rule_is_the_stride_definition ties the two together)
        sel = (np.arange(dims[d]) // stride) % mesh[x] == dev[x]
        shape = [1] * len(dims)
        shape[d] = dims[d]
        own &= sel.reshape(shape)
    return own


def test_owner_rule_is_the_stride_definition():
    for extent, m in ((8, 2), (8, 4), (24, 4), (64, 8)):
        stride = extent // m
        while stride >= 1 and extent % (stride * m) == 0:
            blocks = [oracle.owner(u, stride, m) for u in range(extent)]
            assert blocks == [(u // stride) % m for u in range(extent)]
            # consecutive units of a block share a device; the next block goes to the next device
            assert all(blocks[u] == blocks[u - 1] for u in range(1, extent) if u % stride)
            assert all(blocks[u] == (blocks[u - 1] + 1) % m for u in range(stride, extent, stride))
            stride //= 2


def test_element_level_ownership_on_a_tiny_tensor():
    dims, mesh, eb = (8, 8, 8), (2, 4), 2
    specs = _all_specs(3)
    K = len(specs)
    n_ops = 2
    out_spec = np.array([specs, [0] * K], np.uint32)
    in_spec = np.array([[0] * K, specs], np.uint32)
    # bandwidth 1000 B/us = 1 B/ns: the cost in ns IS the byte count
    R = oracle.build_reshard(mesh, (1000, 1000), (0, 0), np.array([K, K], np.int32), out_spec, in_spec,
                             np.array([list(dims) + [1]], np.int64), np.array([eb], np.int32))

    def axes_of(w):
        res = []
        for x, (state, d, lg) in enumerate(sp.unpack(w)):
            stride = (dims[d] // mesh[x]) >> lg if state == sp.SPLIT else 0
            res.append((state, d, stride))
        return res

    checked = nested = 0
    for a, b in itertools.product(range(K), repeat=2):
        p, q = axes_of(specs[a]), axes_of(specs[b])
        same_dim = lambda s: s[0][0] == sp.SPLIT and s[1][0] == sp.SPLIT and s[0][1] == s[1][1]
        if same_dim(p) or same_dim(q):
            assert R[0, a, b] == INF                        # not a candidate
            continue
        if any(s[0] == sp.PARTIAL for s in p + q):
            continue                                        # partial sums are not an ownership question
        mid = [q[0], p[1]]                                  # axis 0 converted first
        # when producer and consumer swap the dims of the two axes, `mid` splits ONE dim on both axes: a device then
        # holds the units that both per-axis owner rules give it (what `_owned` computes); that layout can be
        # uneven over the devices, and the cost is the exact per-device average like everywhere else
        nested += same_dim(mid)
        per_dev = []
        for dev in itertools.product(range(mesh[0]), range(mesh[1])):
            o_p, o_m, o_q = (_owned(s, dims, mesh, dev) for s in (p, mid, q))
            per_dev.append(((o_m & ~o_p).sum() + (o_q & ~o_m).sum()) * eb)
        # exact per-device average (equal on all devices except for a stride change)
        assert sum(per_dev) % len(per_dev) == 0
        assert R[0, a, b] == sum(per_dev) // len(per_dev), (sp.unpack(specs[a]), sp.unpack(specs[b]))
        checked += 1
    assert checked > 1000 and nested >= 24


def test_swapped_dims_go_through_a_nested_intermediate(golden_dir):
    """Producer splits dim 0 on axis 0 and dim 1 on axis 1, the consumer the other way round.  With axis 0 converted
    first (Sec. 4: sharding is applied per mesh axis) the layout in between has BOTH axes on dim 1: device (k0, k1)
    holds the units u of dim 1 with owner(u, stride_q0, m0) == k0 and owner(u, stride_p1, m1) == k1.  The bytes every
    device receives in the two steps are counted element by element and averaged; the hand-worked figures of the
    fixture (local*(m-1)/m^2 per step) must come out, although the devices' shares differ."""
    row = [r for r in _rows(os.path.join(golden_dir, "reshard_swapped_dims.txt"))][0]
    n, m0, m1, eb, step0, step1 = map(int, row)
    dims, mesh = (n, n, n), (m0, m1)
    p = [(sp.SPLIT, 0, n // m0), (sp.SPLIT, 1, n // m1)]
    q = [(sp.SPLIT, 1, n // m0), (sp.SPLIT, 0, n // m1)]
    mid = [q[0], p[1]]
    got0, got1 = [], []
    for dev in itertools.product(range(m0), range(m1)):
        o_p, o_m, o_q = (_owned(s, dims, mesh, dev) for s in (p, mid, q))
        got0.append(int((o_m & ~o_p).sum()) * eb)
        got1.append(int((o_q & ~o_m).sum()) * eb)
    # the intermediate is a partition of the tensor, but not an even one
    held = [int(_owned(mid, dims, mesh, dev).sum()) for dev in itertools.product(range(m0), range(m1))]
    assert sum(held) == n ** 3 and min(held) == 0 and max(held) == 2 * n ** 3 // (m0 * m1)
    assert sum(got0) == step0 * m0 * m1 and sum(got1) == step1 * m0 * m1
    R = oracle.build_reshard(mesh, (1000, 1000), (0, 0), np.array([1, 1], np.int32),
                             np.array([[sp.word(sp.S_(0), sp.S_(1))], [0]], np.uint32),
                             np.array([[0], [sp.word(sp.S_(1), sp.S_(0))]], np.uint32),
                             np.array([[n, n, n, 1]], np.int64), np.array([eb], np.int32))
    assert R[0, 0, 0] == step0 + step1                     # 1 byte per ns
    assert oracle.axis_bytes(sp.S_(0), sp.S_(1), dims, m0, n ** 3 * eb // m1) == step0
    assert oracle.axis_bytes(sp.S_(1), sp.S_(0), dims, m1, n ** 3 * eb // m0) == step1


def test_invariants_of_the_paper():
    dims, mesh = (16, 64, 32, 16), (4, 8)
    specs = [w for w in _all_specs(4)]
    K = len(specs)
    args = dict(m=mesh, bw_bytes_per_us=(12500, 150000), alpha_ns=(0, 0), K=np.array([K, K], np.int32),
                dims=np.array([list(dims)], np.int64), elem_bytes=np.array([4], np.int32))
    R = oracle.build_reshard(out_spec=np.array([specs, [0] * K], np.uint32),
                             in_spec=np.array([[0] * K, specs], np.uint32), **args)[0]
    valid = np.array([R[j, j] < INF for j in range(K)])
    # matched specs need no communication
    assert all(R[j, j] == 0 for j in range(K) if valid[j])
    assert valid.sum() == K - 4 * 4                         # 4 dims x (2x2 stride pairs) put one dim on both axes
    # replicate -> anything but partial is a local slice
    r = specs.index(sp.word(sp.R_, sp.R_))
    for j in range(K):
        ax = sp.unpack(specs[j])
        if valid[j]:
            assert (R[r, j] == 0) == all(s[0] != sp.PARTIAL for s in ax)
            if any(s[0] == sp.PARTIAL for s in ax):
                assert R[r, j] == INF                       # nothing becomes partial
    # going through "replicate" is never cheaper than resharding directly
    for a, b in itertools.product(range(K), repeat=2):
        if valid[a] and valid[b] and R[a, r] < INF and R[a, b] < INF:
            assert R[a, b] <= R[a, r] + R[r, b]
    # halving every stride (lgdiv 0 -> 1 everywhere) changes no cost
    def bump(w):
        out = 0
        for x, (state, d, lg) in enumerate(sp.unpack(w)):
            out |= sp.axis_byte(state, d, lg + 1 if state == sp.SPLIT else 0) << (8 * x)
        return out
    base = [w for w in specs if all(s[2] == 0 for s in sp.unpack(w))]
    Kb = len(base)
    a0 = dict(args, K=np.array([Kb, Kb], np.int32))
    R0 = oracle.build_reshard(out_spec=np.array([base, [0] * Kb], np.uint32),
                              in_spec=np.array([[0] * Kb, base], np.uint32), **a0)
    R1 = oracle.build_reshard(out_spec=np.array([[bump(w) for w in base], [0] * Kb], np.uint32),
                              in_spec=np.array([[0] * Kb, [bump(w) for w in base]], np.uint32), **a0)
    assert np.array_equal(R0, R1)


def test_padding_latency_and_single_axis():
    dims = np.array([[64, 64, 1, 1]], np.int64)
    specs = [sp.word(sp.S_(0)), sp.word(sp.R_), sp.EMPTY, sp.word(3)]     # empty slot, invalid state
    K = np.array([2, 2], np.int32)
    out_spec = np.array([specs, [0] * 4], np.uint32)
    in_spec = np.array([[0] * 4, specs], np.uint32)
    R = oracle.build_reshard((4,), (1000,), (250,), K, out_spec, in_spec, dims, np.array([1], np.int32))[0]
    assert R[0, 0] == 0 and R[1, 1] == 0 and R[1, 0] == 0
    assert R[0, 1] == 64 * 64 * 3 // 4 + 250               # all-gather bytes at 1 B/ns + latency
    assert np.all(R[2:, :] == INF) and np.all(R[:, 2:] == INF)
    # extents that the mesh axis does not divide make the spec invalid
    bad = oracle.build_reshard((4,), (1000,), (0,), np.array([1, 1], np.int32),
                               np.array([[sp.word(sp.S_(0))], [0]], np.uint32),
                               np.array([[0], [sp.word(sp.R_)]], np.uint32),
                               np.array([[6, 8, 1, 1]], np.int64), np.array([1], np.int32))
    assert bad[0, 0, 0] == INF
    # extents with an odd factor are fine as long as m * 2^lgdiv divides them (hidden 12288 = 3 * 4096)
    assert oracle.axis_bytes(sp.S_(0, 2), sp.S_(0, 0), (12288,), 32, 12288 * 2) == 12288 * 2 * 31 // 1024
