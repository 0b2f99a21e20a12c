"""Synthetic cones and their packing into one chain batch (host side, numpy).

A cone (Sec. 4.3.2 of the paper, level 1) is one root operator with several
inputs whose other nodes have one input each, so every branch is a chain that
ends in the root.  `random_cones` draws seeded cones; `pack` lays all branches
of all cones out as ONE batch for the chain DP: every branch gets the root
appended as its last operator with cost 0, and shorter branches are padded in
front with zero-cost operators joined by identity tables (0 on the diagonal,
INF elsewhere), which leave the branch's costs unchanged.  Input marshalling
only; no cost is minimised here.
"""
from __future__ import annotations

import numpy as np

from .synthetic import BASE_SEED, INF


def random_cones(n_cones: int, K: int, max_branches: int = 4, max_len: int = 6, c_range: int = 2000,
                 r_range: int = 10000, seed: int = BASE_SEED, infeasible: float = 0.0):
    """-> list of (branches, c_root); branches = list of (c[len][K], R[len][K][K]), last R = edge into the root."""
    rng = np.random.default_rng(seed)
    cones = []
    for _ in range(n_cones):
        branches = []
        for _ in range(int(rng.integers(1, max_branches + 1))):
            n = int(rng.integers(1, max_len + 1))
            cb = rng.integers(0, c_range, size=(n, K)).astype(np.int64)
            Rb = rng.integers(0, r_range, size=(n, K, K)).astype(np.int64)
            d = np.arange(K)
            Rb[:, d, d] = 0
            if infeasible > 0:
                Rb[rng.random(Rb.shape) < infeasible] = INF
            branches.append((cb, Rb))
        cones.append((branches, rng.integers(0, c_range, size=K).astype(np.int64)))
    return cones


def pack(cones, Kp: int):
    """-> dict(c[Bb][N][Kp], R[Bb][N-1][Kp][Kp], branch_start int32[n_cones+1], c_root[n_cones][Kp], lens, N)
    with N = longest branch + 1 (the root)."""
    K = cones[0][1].shape[0]
    lens = [cb.shape[0] for branches, _ in cones for cb, _ in branches]
    N = max(lens) + 1
    Bb = len(lens)
    c = np.zeros((Bb, N, Kp), dtype=np.int64)
    R = np.full((Bb, N - 1, Kp, Kp), INF, dtype=np.int64)
    d = np.arange(Kp)
    R[:, :, d, d] = 0                                   # identity tables; real ones overwrite them below
    c_root = np.full((len(cones), Kp), INF, dtype=np.int64)
    start = np.zeros(len(cones) + 1, dtype=np.int32)
    b = 0
    for q, (branches, cr) in enumerate(cones):
        c_root[q, :K] = cr
        for cb, Rb in branches:
            n = cb.shape[0]
            off = N - 1 - n                             # padding operators in front
            c[b, off:N - 1, :K] = cb
            c[b, off:N - 1, K:] = INF                   # empty candidate slots of real operators
            R[b, off:, :, :] = INF
            R[b, off:, :K, :K] = Rb
            # the root (last operator) costs 0 here; its empty slots stay unreachable through R
            b += 1
        start[q + 1] = b
    return dict(c=c, R=R, branch_start=start, c_root=c_root, lens=np.array(lens, dtype=np.int32), N=N, Kp=Kp)
