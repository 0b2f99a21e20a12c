"""Seeded synthetic search inputs (host side, numpy).

These generators produce the *inputs* of plan scoring -- node cost tables,
edge cost tables, segment costs -- and nothing of the method itself.  Both the
CPU oracle's tests and the GPU tests draw from here, so that the two sides see
identical numbers without sharing any arithmetic of the method.

Random numbers come from one counter-based generator, SplitMix64 (Steele,
Lea, Flood, "Fast splittable pseudorandom number generators", OOPSLA 2014) in
random-access form: the n-th output of the generator seeded with s is
mix64(s + (n+1)*GOLDEN).  A device-side fill kernel implements the same
definition for tables that are too large to upload; a GPU test compares the
two element by element.
"""
from __future__ import annotations

import numpy as np

INF = np.int64(1) << np.int64(52)          # "infeasible" marker of the cost tables
BASE_SEED = 20230216

GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_M1 = np.uint64(0xBF58476D1CE4E5B9)
_M2 = np.uint64(0x94D049BB133111EB)

TAG_NODE = 1      # stream of node-cost tables c
TAG_EDGE = 2      # stream of edge-cost tables R
TAG_SEG = 3       # stream of pipeline segment costs


def mix64(z):
    """SplitMix64 output function on uint64 (scalar or array), wrapping."""
    z = np.asarray(z, dtype=np.uint64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> np.uint64(30))) * _M1
        z = (z ^ (z >> np.uint64(27))) * _M2
        return z ^ (z >> np.uint64(31))


def stream_seed(seed: int, problem, tag: int):
    """Seed of the stream that fills table `tag` of problem `problem`."""
    with np.errstate(over="ignore"):
        p = np.asarray(problem, dtype=np.uint64)
        s = mix64(np.uint64(seed) + (p + np.uint64(1)) * GOLDEN)
        return mix64(s + np.uint64(tag) * GOLDEN)


def uniform_at(sseed, idx, rng: int):
    """Values in [0, rng) at positions idx of the stream seeded sseed (rng <= 2^32)."""
    assert 0 < rng <= (1 << 32)
    with np.errstate(over="ignore"):
        idx = np.asarray(idx, dtype=np.uint64)
        z = mix64(np.asarray(sseed, dtype=np.uint64) + (idx + np.uint64(1)) * GOLDEN)
        return (((z >> np.uint64(32)) * np.uint64(rng)) >> np.uint64(32)).astype(np.int64)


def pad_k(x: np.ndarray, Kp: int, axes) -> np.ndarray:
    """Pad the given axes of x to length Kp with INF (empty candidate slots)."""
    pads = [(0, 0)] * x.ndim
    for ax in axes:
        pads[ax] = (0, Kp - x.shape[ax])
    return np.pad(x, pads, constant_values=INF)


def random_chain_problem(problem: int, N: int, K: int, c_range: int, r_range: int,
                         seed: int = BASE_SEED, c_lo: int = 0, zero_diag: bool = True):
    """One chain problem: c[N][K] in [c_lo, c_lo+c_range), R[N-1][K][K] in [0, r_range).

    Element (i, j) of c is position i*K+j of the node stream; element (i, a, b)
    of R is position (i*K+a)*K+b of the edge stream; R[i][a][a] = 0.
    """
    sc = stream_seed(seed, problem, TAG_NODE)
    sr = stream_seed(seed, problem, TAG_EDGE)
    c = uniform_at(sc, np.arange(N * K, dtype=np.uint64), c_range).reshape(N, K) + c_lo
    R = uniform_at(sr, np.arange((N - 1) * K * K, dtype=np.uint64), r_range).reshape(N - 1, K, K)
    if zero_diag and N > 1:
        d = np.arange(K)
        R[:, d, d] = 0
    return c, R


def random_chain_batch(problems, N: int, K: int, c_range: int, r_range: int,
                       seed: int = BASE_SEED, Kp: int | None = None, c_lo: int = 0):
    """Stack of problems (by problem id), padded to Kp: c[B][N][Kp], R[B][N-1][Kp][Kp]."""
    Kp = K if Kp is None else Kp
    cs, Rs = [], []
    for p in problems:
        c, R = random_chain_problem(int(p), N, K, c_range, r_range, seed, c_lo)
        cs.append(pad_k(c, Kp, (1,)))
        Rs.append(pad_k(R, Kp, (1, 2)))
    return np.ascontiguousarray(np.stack(cs)), np.ascontiguousarray(np.stack(Rs))


def segment_costs(problem: int, L: int, lo: int = 1, hi: int = 100000, seed: int = BASE_SEED):
    """Pipeline segment costs, int64 uniform in [lo, hi)."""
    s = stream_seed(seed, problem, TAG_SEG)
    return uniform_at(s, np.arange(L, dtype=np.uint64), hi - lo) + lo


# The five named workloads (sizes only; see the builders above and in specs.py).
TINY_CHAIN = dict(B=1, N=10, K=4, c_range=1000, r_range=5000)
BATCHED_CHAINS = dict(B=4096, N=512, K=128, c_range=1_000_000, r_range=10_000_000)
STAGE_PARTITION = dict(L=4096, S=64, lo=1, hi=100000, seg_ops=8, seg_K=64,
                       seg_c_lo=1, seg_c_range=1999, seg_r_range=10000)
