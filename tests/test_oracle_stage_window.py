"""Pins of the windowed pipeline-stage oracle (CPU only).

Sec. 5.1: tensors crossing a stage boundary are transferred; Sec. 5.2: every
operator stays within a tolerance eps of the stage perfect balance gives it
(time_per_stage = total / d).  Checked against enumeration of all cut sets with
the per-segment bounds evaluated in exact rational arithmetic, and against the
plain stage oracle when the bounds are off and nothing is transferred.
"""
import itertools
import math
from fractions import Fraction

import numpy as np
import pytest

import oracle

INF = oracle.INF


def enumerate_cuts(cost, xfer, d, eps):
    """min over cut sets of the max stage time, segments checked one by one against their bounds."""
    L = len(cost)
    P = [0]
    for x in cost:
        P.append(P[-1] + int(x))
    tps = Fraction(P[L], d)
    best = None
    for cuts in itertools.combinations(range(1, L), d - 1):
        b = (0,) + cuts + (L,)
        ok = True
        if eps is not None and P[L] > 0:
            for t in range(d):
                for l in range(b[t], b[t + 1]):
                    start = Fraction(P[l]) / tps
                    if not (math.floor(start - eps) <= t <= math.ceil(start + eps)):
                        ok = False
        if not ok:
            continue
        m = max(P[b[t + 1]] - P[b[t]] + (int(xfer[b[t]]) if t > 0 else 0) for t in range(d))
        best = m if best is None or m < best else best
    return INF if best is None else best


@pytest.mark.parametrize("seed", range(10))
def test_against_all_cut_sets(seed):
    rng = np.random.default_rng(seed)
    L = int(rng.integers(2, 12))
    d = int(rng.integers(1, min(L, 5) + 1))
    cost = rng.integers(0 if seed % 3 == 0 else 1, 30, size=L).astype(np.int64)
    xfer = rng.integers(0, 20, size=L + 1).astype(np.int64)
    for num, den in ((-1, 1), (0, 1), (1, 4), (1, 2), (1, 1), (3, 2)):
        eps = None if num < 0 else Fraction(num, den)
        want = enumerate_cuts(cost, xfer, d, eps)
        bott, cut, bounds = oracle.stage_window(cost[None], d, xfer[None], num, den)
        assert bott[0] == want, (num, den)
        if want < INF:
            b = bounds[0]
            assert b[0] == 0 and b[-1] == L and np.all(np.diff(b) >= 1)
            P = np.concatenate([[0], np.cumsum(cost)])
            assert max(P[b[t + 1]] - P[b[t]] + (xfer[b[t]] if t > 0 else 0) for t in range(d)) == want
        else:
            assert np.all(bounds[0] == -1)


@pytest.mark.parametrize("L,d", [(40, 5), (97, 16)])
def test_reduces_to_the_plain_stage_dp(L, d):
    rng = np.random.default_rng(L)
    cost = rng.integers(1, 1000, size=(2, L)).astype(np.int64)
    plain_bott, plain_cut, plain_bounds = oracle.stage_dp(cost, d, s_query=d)
    bott, cut, bounds = oracle.stage_window(cost, d, None, -1, 1)
    assert np.array_equal(bott, plain_bott[:, d - 1]) and np.array_equal(bounds, plain_bounds)
    assert np.array_equal(cut, plain_cut)
    # a huge tolerance is no constraint; tightening it never helps
    wide, _, _ = oracle.stage_window(cost, d, None, 1000, 1)
    assert np.array_equal(wide, bott)
    last = bott
    for num, den in ((2, 1), (1, 1), (1, 2), (1, 8), (0, 1)):
        b, _, _ = oracle.stage_window(cost, d, None, num, den)
        assert np.all(b >= last)
        last = b
    # transfers only ever add time
    xfer = rng.integers(0, 500, size=(2, L + 1)).astype(np.int64)
    with_x, _, _ = oracle.stage_window(cost, d, xfer, -1, 1)
    assert np.all(with_x >= bott) and np.all(with_x <= bott + xfer.max())
