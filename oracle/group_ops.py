"""Oracle for the group-level operators of the DBuffer other than the plain copy.
TEST INFRASTRUCTURE ONLY - never imported by the product.

Section 5 ("Distributed Buffer") names the per-tensor kernels that run around a
collective - add, scale, zero, copy - and fuses each across the tensors of a group.  Copy
and zero are ragged_pack; the others are defined here on the bf16 buffer of m*S elements
in which tensor t owns [l_t, l_t + e_t) and everything else is padding:

  group_zero    every element of the buffer becomes +0
  group_scale   DB[l_t + i] <- bf16( f32(DB[l_t + i]) * alpha )          (gradient pre- or
                post-division); padding is not touched and stays +0
  group_add     DB[l_t + i] <- bf16( f32(DB[l_t + i]) + alpha * f32(src_t[i]) )
                (accumulation of a new set of per-tensor gradients into the buffer);
                padding is not touched
  pack_scaled   DB[l_t + i] <- bf16( f32(src_t[i]) * alpha ), padding +0: copy-in and
                pre-division in one pass

The paper gives no arithmetic for them; the reading taken: alpha is an fp32 number, every
product and sum is a single correctly rounded fp32 operation in the order written (no fused
multiply-add), and the result is rounded to bf16 once, to nearest even.  bf16 values
travel as uint16 bit patterns.
"""
from __future__ import annotations

from typing import Sequence

import numpy as np

from .dbuffer import bf16_bits_to_f32


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest, ties to the even mantissa (finite inputs)."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    keep = (u >> np.uint64(16)) & np.uint64(1)
    return ((u + np.uint64(0x7FFF) + keep) >> np.uint64(16)).astype(np.uint16)


def group_zero(total: int) -> np.ndarray:
    return np.zeros(total, dtype=np.uint16)


def group_scale(db: np.ndarray, offsets: Sequence[int], sizes: Sequence[int], alpha: float) -> np.ndarray:
    a = np.float32(alpha)
    out = np.array(db, dtype=np.uint16, copy=True)
    for l, e in zip(offsets, sizes):
        x = bf16_bits_to_f32(out[l:l + e])
        out[l:l + e] = f32_to_bf16_bits(x * a)
    return out


def group_add(db: np.ndarray, srcs: Sequence[np.ndarray], offsets: Sequence[int], alpha: float) -> np.ndarray:
    a = np.float32(alpha)
    out = np.array(db, dtype=np.uint16, copy=True)
    for src, l in zip(srcs, offsets):
        flat = np.asarray(src, dtype=np.uint16).reshape(-1)
        term = a * bf16_bits_to_f32(flat)                      # fp32 product, rounded
        acc = bf16_bits_to_f32(out[l:l + flat.size]) + term    # fp32 sum, rounded
        out[l:l + flat.size] = f32_to_bf16_bits(acc)
    return out


def pack_scaled(srcs: Sequence[np.ndarray], offsets: Sequence[int], total: int, alpha: float) -> np.ndarray:
    a = np.float32(alpha)
    db = np.zeros(total, dtype=np.uint16)
    for src, l in zip(srcs, offsets):
        flat = np.asarray(src, dtype=np.uint16).reshape(-1)
        db[l:l + flat.size] = f32_to_bf16_bits(bf16_bits_to_f32(flat) * a)
    return db
