"""Synthetic in-trees of operators (host side, numpy).

An in-tree: every operator feeds exactly one consumer (its parent) and may have
several inputs; the root feeds nobody.  This is a cone of the paper (Sec. 4.3.2,
level 1) whose inner nodes may join several inputs as well.  Nodes are numbered
so that parent[i] > i and a node whose only input is its predecessor continues
that input's run (so that runs of single-input nodes are consecutive, like the
operators of a chain).  Input marshalling only; no cost is minimised here.
"""
from __future__ import annotations

import numpy as np

from .synthetic import BASE_SEED, INF


def random_tree(n: int, max_fan_in: int = 4, chain_bias: float = 0.6, seed: int = BASE_SEED) -> np.ndarray:
    """parent int32[n] of a seeded random in-tree with parent[i] > i, root n-1 (parent -1).  A node takes its
    predecessor's place in a run with probability chain_bias, otherwise a later node that still has room."""
    rng = np.random.default_rng(seed)
    parent = np.full(n, -1, dtype=np.int32)
    fan = np.zeros(n, dtype=np.int64)
    for i in range(n - 2, -1, -1):                       # choose who consumes node i
        if rng.random() < chain_bias and fan[i + 1] < max_fan_in:
            p = i + 1
        else:
            room = [j for j in range(i + 1, n) if fan[j] < max_fan_in]
            p = int(rng.choice(room)) if room else n - 1
        parent[i] = p
        fan[p] += 1
    return parent


def random_tree_costs(parent: np.ndarray, K: int, Kp: int | None = None, c_range: int = 2000, r_range: int = 10000,
                      seed: int = BASE_SEED, infeasible: float = 0.0, ragged: bool = False):
    """-> c[n][Kp], R[n-1][Kp][Kp]: node costs and the table of every edge i -> parent[i] (row = strategy of i)."""
    rng = np.random.default_rng(seed + 1)
    n = parent.shape[0]
    Kp = K if Kp is None else Kp
    c = np.full((n, Kp), INF, dtype=np.int64)
    R = np.full((max(n - 1, 0), Kp, Kp), INF, dtype=np.int64)
    Ki = rng.integers(max(1, K // 2), K + 1, size=n) if ragged else np.full(n, K)
    for i in range(n):
        c[i, :Ki[i]] = rng.integers(0, c_range, size=Ki[i])
        if i < n - 1:
            kp = Ki[parent[i]]
            R[i, :Ki[i], :kp] = rng.integers(0, r_range, size=(Ki[i], kp))
    if infeasible > 0:
        R[rng.random(R.shape) < infeasible] = INF
        dead = rng.random(c.shape) < infeasible / 2
        dead[:, 0] = False
        c[dead] = INF
    return c, R


def depth(parent: np.ndarray) -> int:
    """Edges on the longest path from a leaf to the root."""
    n = parent.shape[0]
    h = np.zeros(n, dtype=np.int64)
    for i in range(n - 1):
        h[parent[i]] = max(h[parent[i]], h[i] + 1)
    return int(h[n - 1])
