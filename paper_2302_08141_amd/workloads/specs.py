"""Sharding-spec words: the input format of the reshard builder.

A spec describes how one tensor is laid out on a logical device mesh of one
or two axes.  Per mesh axis one byte:

    bits 0..1  state  0 = replicate, 1 = split, 2 = partial (full shape, partial sums)
    bits 2..4  dim    tensor dimension that is split (0..3), 0 unless state = split
    bits 5..7  lgdiv  stride = (extent[dim] / axis_size) >> lgdiv; 0 = maximum stride

(the (dim, stride) pair, replicate and partial of Sec. 4.1 and Sec. 4.3.3 of the
paper; the mesh axes are sharded independently, Sec. 4).  Axis 0 sits in bits
0..7 of the uint32 word, axis 1 in bits 8..15.  EMPTY marks an unused slot.
This module only packs and unpacks words; it computes no cost.
"""
from __future__ import annotations

REPLICATE, SPLIT, PARTIAL = 0, 1, 2
EMPTY = 0xFFFFFFFF


def axis_byte(state: int, dim: int = 0, lgdiv: int = 0) -> int:
    assert 0 <= state <= 3 and 0 <= dim <= 7 and 0 <= lgdiv <= 7
    if state != SPLIT:
        dim, lgdiv = 0, 0
    return state | (dim << 2) | (lgdiv << 5)


R_ = axis_byte(REPLICATE)
P_ = axis_byte(PARTIAL)


def S_(dim: int, lgdiv: int = 0) -> int:
    return axis_byte(SPLIT, dim, lgdiv)


def word(axis0: int, axis1: int = R_) -> int:
    return (axis0 & 0xFF) | ((axis1 & 0xFF) << 8)


def unpack(w: int):
    """-> [(state, dim, lgdiv) per axis]"""
    return [((w >> (8 * x)) & 3, (w >> (8 * x + 2)) & 7, (w >> (8 * x + 5)) & 7) for x in range(2)]
