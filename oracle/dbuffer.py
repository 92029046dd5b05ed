"""Oracle for the DBuffer data movement: ragged_pack, its inverse, and shard_reduce.
TEST INFRASTRUCTURE ONLY - never imported by the product.

bf16 values travel as uint16 bit patterns so that copies are compared bit for bit.

ragged_pack / unpack_bf16: the group-level copy and zero operators of the DBuffer
(Section 5, "Distributed Buffer"), with each tensor at its planned interval [l_t, r_t)
of the rank-major buffer of m*S elements; everything outside the intervals is padding
and holds +0.

shard_reduce: the arithmetic of the gradient ReduceScatter (Section 2.3: gradients of a
unit are reduced back across devices) as seen by one device: the W partial copies of
its own region are summed, then averaged.  The definition is evaluated in float64.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 -> fp32 is exact: the 16 bits are the top half of the fp32 pattern."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def ragged_pack(srcs: Sequence[np.ndarray], offsets: Sequence[int], total: int) -> np.ndarray:
    """DB = zeros(m*S); DB[l_t : l_t + e_t] = src_t (flattened, row-major)."""
    db = np.zeros(total, dtype=np.uint16)
    for src, l in zip(srcs, offsets):
        flat = np.asarray(src, dtype=np.uint16).reshape(-1)
        db[l:l + flat.size] = flat
    return db


def unpack_bf16(db: np.ndarray, offsets: Sequence[int], sizes: Sequence[int]) -> List[np.ndarray]:
    """Inverse slice: tensor t = DB[l_t : l_t + e_t]."""
    return [db[l:l + e].copy() for l, e in zip(offsets, sizes)]


def shard_reduce(partials: np.ndarray, segments: Sequence[Tuple[int, int, int, int]]) -> np.ndarray:
    """out[i] = (1/W) * sum_w P[w][i] on the payload of the region, 0 on its padding.

    partials: (W, S) uint16 bf16 bits - partial w's copy of this rank's region.
    segments: the rank's (t, src_off, dst_off, n) list; dst_off/n mark the payload.
    Sum and division in float64, result rounded once to fp32."""
    W, S = partials.shape
    out = np.zeros(S, dtype=np.float32)
    for _, _, d, n in segments:
        acc = np.zeros(n, dtype=np.float64)
        for w in range(W):
            acc += bf16_bits_to_f32(partials[w, d:d + n]).astype(np.float64)
        out[d:d + n] = (acc / W).astype(np.float32)
    return out


def shard_reduce_f32_ordered(partials: np.ndarray, segments: Sequence[Tuple[int, int, int, int]]) -> np.ndarray:
    """The same mean evaluated in fp32 in one stated order, for bit-for-bit reproducibility
    of the reduction (a reading: the paper fixes no order; any fixed one is a valid
    ReduceScatter):  partial w is added, in increasing w, to running sum number (w mod 8),
    each sum starting from +0; the eight sums a0..a7 are combined as
    ((a0 + a1) + (a2 + a3)) + ((a4 + a5) + (a6 + a7)); the result is multiplied by the fp32
    value of 1/W.  Every operation is a single rounded fp32 operation."""
    W, S = partials.shape
    out = np.zeros(S, dtype=np.float32)
    inv = np.float32(1.0) / np.float32(W)
    for _, _, d, n in segments:
        a = [np.zeros(n, dtype=np.float32) for _ in range(8)]
        for w in range(W):
            a[w % 8] = a[w % 8] + bf16_bits_to_f32(partials[w, d:d + n])
        total = ((a[0] + a[1]) + (a[2] + a[3])) + ((a[4] + a[5]) + (a[6] + a[7]))
        out[d:d + n] = total * inv
    return out


def shard_reduce_abs_sum(partials: np.ndarray) -> np.ndarray:
    """sum_w |P[w][i]| in float64: the scale of the accepted error of shard_reduce."""
    W, S = partials.shape
    acc = np.zeros(S, dtype=np.float64)
    for w in range(W):
        acc += np.abs(bf16_bits_to_f32(partials[w]).astype(np.float64))
    return acc
