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


def strided_region_starts(m: int, S: int, groups: int, group: int) -> List[int]:
    """Where the m rank regions of one DBuffer sit inside a buffer gathered over a 2-D device
    mesh (Section 4, composing RaggedShard with Shard(0) of expert / tensor parallelism: the
    parameter is first split over `groups` devices of the other mesh dimension, then each part is
    ragged-sharded over m devices).  Reading taken for the "stride metadata" of StridedRaggedShard:
    the gathered buffer holds the regions device-major, FSDP rank outermost, so region k of group
    `group` starts at element (k * groups + group) * S - a regular stride of groups * S."""
    return [(k * groups + group) * S for k in range(m)]


def unpack_bf16_strided(buf: np.ndarray, offsets: Sequence[int], sizes: Sequence[int], S: int,
                        starts: Sequence[int]) -> List[np.ndarray]:
    """Tensor t = the elements at logical buffer positions [l_t, l_t + e_t), where logical position
    x lives at buf[starts[x // S] + x % S]: the reshuffle that materialises the tensors of one
    group from the mesh-ordered gathered buffer."""
    out = []
    for l, e in zip(offsets, sizes):
        t = np.empty(e, dtype=np.uint16)
        x = l
        while x < l + e:
            k, j = divmod(x, S)
            n = min(S - j, l + e - x)
            t[x - l:x - l + n] = buf[starts[k] + j:starts[k] + j + n]
            x += n
        out.append(t)
    return out


def ragged_pack_strided(buf: np.ndarray, srcs: Sequence[np.ndarray], offsets: Sequence[int], S: int,
                        starts: Sequence[int]) -> np.ndarray:
    """The inverse placement into a copy of `buf`: every region listed in `starts` is zeroed and
    then receives its part of the tensors; the rest of the buffer (other groups' regions) is kept."""
    out = np.array(buf, dtype=np.uint16, copy=True)
    for st in starts:
        out[st:st + S] = 0
    for src, l in zip(srcs, offsets):
        flat = np.asarray(src, dtype=np.uint16).reshape(-1)
        x = l
        while x < l + flat.size:
            k, j = divmod(x, S)
            n = min(S - j, l + flat.size - x)
            out[starts[k] + j:starts[k] + j + n] = flat[x - l:x - l + n]
            x += n
    return out


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
