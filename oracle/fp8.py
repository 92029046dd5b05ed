"""Oracle for block-wise FP8 quantisation of a ragged shard and its inverse.
TEST INFRASTRUCTURE ONLY - never imported by the product.

The paper motivates communication-free block-wise quantisation (Section 2.1
"Block-wise Quantization", Section 4 "Block-wise RaggedShard", Section 6.4: the
128-row granularity reproduces 128x128 tiling) but gives no number format; the
numerics here are the build's stated reading:

  format   OCP FP8 E4M3 ("fn"): 1 sign, 4 exponent (bias 7), 3 mantissa bits, no
           infinities, NaN = S.1111.111, largest finite 0x7E = 448.
           value(E = 0) = +-(M/8) * 2^-6 ;  value(E > 0) = +-(1 + M/8) * 2^(E-7)
  block    128x128 tiles of a 2-D tensor (edge tiles may be partial), or 1x128 runs
           along each row of a 2-D tensor / along a 1-D tensor
  step 1   x32 = fp32(x_bf16) (exact);  amax = max |x32| over the block's valid elements
  step 2   scale = amax / 448 in fp32 (one correctly rounded division)
  step 3   amax == 0: codes 0x00, scale 0.  Otherwise y = x32 / scale (correctly rounded
           fp32 division), y clamped to [-448, 448], code = nearest E4M3 value to y,
           ties to the even mantissa, sign bit kept (also for results that round to 0)
  step 4   dequantise: v = value(code) * scale (one fp32 multiply), out = bf16 RNE of v

Scales of a unit form one flat fp32 array in buffer order: tensor-major, then block row,
then block column.
"""
from __future__ import annotations

from typing import List, Tuple

import numpy as np

from .dbuffer import bf16_bits_to_f32
from .plan import BLOCK_128x128, BLOCK_1x128, Plan, TensorSpec

E4M3_MAX = np.float32(448.0)


def e4m3_value(code: int) -> float:
    """The real number a code denotes (format definition above); NaN codes give nan."""
    s, E, M = code >> 7, (code >> 3) & 0xF, code & 7
    if E == 0xF and M == 7:
        return float("nan")
    mag = (M / 8.0) * 2.0 ** -6 if E == 0 else (1.0 + M / 8.0) * 2.0 ** (E - 7)
    return -mag if s else mag


def decode_table() -> np.ndarray:
    """value(code) for all 256 codes as fp32 (every finite value is exact in fp32)."""
    return np.array([e4m3_value(c) for c in range(256)], dtype=np.float32)


_POS = np.array([e4m3_value(c) for c in range(0x7F)], dtype=np.float64)   # 0 .. 448, ascending
_MID = (_POS[:-1] + _POS[1:]) / 2.0                                      # exact in fp64


def encode_e4m3(y: np.ndarray) -> np.ndarray:
    """Nearest-value encoding with ties to even of fp32 values already within [-448, 448]."""
    y = np.asarray(y, dtype=np.float32)
    a = np.abs(y).astype(np.float64)
    assert not np.any(a > 448.0), "encode_e4m3 expects clamped input"
    idx = np.searchsorted(_MID, a, side="left")          # number of midpoints strictly below a
    # a lies in (MID[idx-1], MID[idx]]: nearest is code idx, unless a == MID[idx] (a tie
    # between idx and idx+1), which goes to whichever code has an even mantissa (even code)
    tie = (idx < _MID.size) & (a == _MID[np.minimum(idx, _MID.size - 1)])
    idx = np.where(tie & (idx % 2 == 1), idx + 1, idx)
    return (idx.astype(np.uint8) | (np.signbit(y).astype(np.uint8) << 7)).astype(np.uint8)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns, round to nearest even (finite inputs)."""
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    return ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)


def _as_2d(spec: TensorSpec) -> Tuple[int, int, int, int]:
    """(R, C, block height, block width) of the tensor viewed as rows of quant blocks."""
    if spec.cols == 0:
        return 1, spec.rows, 1, 128
    if spec.mode == BLOCK_128x128:
        return spec.rows, spec.cols, 128, 128
    if spec.mode == BLOCK_1x128:
        return spec.rows, spec.cols, 1, 128
    raise ValueError("tensor is not quantised")


def quantise_matrix_f32(x: np.ndarray, bh: int, bw: int) -> Tuple[np.ndarray, np.ndarray]:
    """Steps 1-3 on an (R, C) matrix of fp32 values with bh x bw blocks.
    Returns codes (R, C) uint8 and scales (ceil(R/bh), ceil(C/bw)) fp32.
    A block is live when its scale is non-zero.  For bf16 inputs that is the same as amax > 0
    (the smallest bf16 magnitude over 448 is still a non-zero fp32); an fp32 input below 2^-140
    can have its scale underflow to zero, and such a block is stored like an all-zero one."""
    x = np.asarray(x, dtype=np.float32)
    R, C = x.shape
    nbr, nbc = -(-R // bh), -(-C // bw)
    codes = np.empty((R, C), dtype=np.uint8)
    scales = np.empty((nbr, nbc), dtype=np.float32)
    for br in range(nbr):
        rows = x[br * bh:(br + 1) * bh]                       # (h, C), h <= bh
        h = rows.shape[0]
        # zero-extend the last partial block: zeros never change max|x|
        wide = np.zeros((h, nbc * bw), dtype=np.float32)
        wide[:, :C] = rows
        blk = wide.reshape(h, nbc, bw)
        amax = np.abs(blk).max(axis=(0, 2)).astype(np.float32)   # (nbc,)
        scale = amax / E4M3_MAX                                   # fp32 / fp32
        live = scale > 0
        safe = np.where(live, scale, np.float32(1.0))
        y = blk / safe[None, :, None]                             # fp32 / fp32
        y = np.clip(y, -E4M3_MAX, E4M3_MAX)
        c = encode_e4m3(y)
        c = np.where(live[None, :, None], c, np.uint8(0))
        codes[br * bh:(br + 1) * bh] = c.reshape(h, nbc * bw)[:, :C]
        scales[br] = np.where(live, scale, np.float32(0.0))
    return codes, scales


def quantise_matrix(bits: np.ndarray, bh: int, bw: int) -> Tuple[np.ndarray, np.ndarray]:
    """Steps 1-3 on an (R, C) matrix of bf16 bits with bh x bw blocks."""
    return quantise_matrix_f32(bf16_bits_to_f32(bits), bh, bw)


def quantise_tensor(bits: np.ndarray, spec: TensorSpec) -> Tuple[np.ndarray, np.ndarray]:
    """codes (flat, e_t) and scales (flat, block-row-major) of one whole tensor."""
    R, C, bh, bw = _as_2d(spec)
    codes, scales = quantise_matrix(np.asarray(bits, dtype=np.uint16).reshape(R, C), bh, bw)
    return codes.reshape(-1), scales.reshape(-1)


def dequantise_tensor(codes: np.ndarray, scales: np.ndarray, spec: TensorSpec) -> np.ndarray:
    """Step 4 for one tensor: bf16 bits (flat) from its codes and its scales."""
    R, C, bh, bw = _as_2d(spec)
    nbr, nbc = -(-R // bh), -(-C // bw)
    tab = decode_table()
    cod = np.asarray(codes, dtype=np.uint8).reshape(R, C)
    sc = np.asarray(scales, dtype=np.float32).reshape(nbr, nbc)
    out = np.empty((R, C), dtype=np.uint16)
    for br in range(nbr):
        rows = cod[br * bh:(br + 1) * bh]
        h = rows.shape[0]
        wide = np.zeros((h, nbc * bw), dtype=np.uint8)
        wide[:, :C] = rows
        v = tab[wide].reshape(h, nbc, bw) * sc[br][None, :, None]      # fp32 * fp32
        out[br * bh:(br + 1) * bh] = f32_to_bf16_bits(v).reshape(h, nbc * bw)[:, :C]
    return out.reshape(-1)


def dequantise_tensor_f32(codes: np.ndarray, scales: np.ndarray, spec: TensorSpec) -> np.ndarray:
    """Step 4 without the final rounding: fp32 value(code) * scale (one fp32 multiply), flat.
    The form an fp32 master copy of the gathered parameters takes."""
    R, C, bh, bw = _as_2d(spec)
    nbr, nbc = -(-R // bh), -(-C // bw)
    tab = decode_table()
    cod = np.asarray(codes, dtype=np.uint8).reshape(R, C)
    sc = np.asarray(scales, dtype=np.float32).reshape(nbr, nbc)
    out = np.empty((R, C), dtype=np.float32)
    for br in range(nbr):
        rows = cod[br * bh:(br + 1) * bh]
        h = rows.shape[0]
        wide = np.zeros((h, nbc * bw), dtype=np.uint8)
        wide[:, :C] = rows
        v = tab[wide].reshape(h, nbc, bw) * sc[br][None, :, None]      # fp32 * fp32
        out[br * bh:(br + 1) * bh] = v.reshape(h, nbc * bw)[:, :C]
    return out.reshape(-1)


def block_quant_all(plan: Plan, db: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """Quantise every tensor of the packed unit as a whole.  codes: m*S uint8 at the same
    element offsets as db (padding 0x00); scales: the unit's flat scale array."""
    codes = np.zeros(plan.total, dtype=np.uint8)
    scales = np.zeros(plan.scale_bases()[-1], dtype=np.float32)
    for spec, l, sb in zip(plan.specs, plan.offsets, plan.scale_bases()):
        if not spec.quantised:
            continue
        c, s = quantise_tensor(db[l:l + spec.e], spec)
        codes[l:l + spec.e] = c
        scales[sb:sb + s.size] = s
    return codes, scales


def block_quant_shard(plan: Plan, k: int, region: np.ndarray, f32: bool = False) -> Tuple[np.ndarray, np.ndarray]:
    """Quantise rank k's region using nothing but that region (the point of keeping blocks
    whole on a rank: no scale exchange).  Each segment is a run of whole granules, i.e.
    whole rows of quantisation blocks, and is quantised as a tensor of its own.
    region: bf16 bits, or (f32) fp32 values.  Returns codes (S,) and the rank's slice of the
    scale array."""
    codes = np.zeros(plan.S, dtype=np.uint8)
    out_scales = []
    for t, src_off, dst_off, n in plan.rank_segments(k):
        spec = plan.specs[t]
        if not spec.quantised:
            continue
        if spec.cols == 0:
            assert src_off % 128 == 0
            sub = TensorSpec(n, 0, spec.mode)
        else:
            assert src_off % spec.g == 0 and n % spec.cols == 0
            sub = TensorSpec(n // spec.cols, spec.cols, spec.mode)
        if f32:
            R, C, bh, bw = _as_2d(sub)
            c, s = quantise_matrix_f32(np.asarray(region[dst_off:dst_off + n], dtype=np.float32).reshape(R, C),
                                       bh, bw)
            c, s = c.reshape(-1), s.reshape(-1)
        else:
            c, s = quantise_tensor(region[dst_off:dst_off + n], sub)
        codes[dst_off:dst_off + n] = c
        out_scales.append(s)
    sc = np.concatenate(out_scales) if out_scales else np.zeros(0, dtype=np.float32)
    return codes, sc.astype(np.float32)


def reduce_quant_shard(plan: Plan, k: int, partials: np.ndarray) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """The fused form of the two steps on rank k: the fp32 mean of the partials (W, S) of bf16
    bits in the stated summation order, zero on padding, and that mean quantised block by
    block without passing through bf16.  Returns (codes, scales, mean)."""
    from .dbuffer import shard_reduce_f32_ordered
    mean = shard_reduce_f32_ordered(partials, plan.rank_segments(k))
    codes, scales = block_quant_shard(plan, k, mean, f32=True)
    return codes, scales, mean


def gather_strided_codes(plan: Plan, buf: np.ndarray, starts) -> np.ndarray:
    """The logical code buffer (m * S) of one group of a buffer gathered over a 2-D device mesh:
    logical position x lives at buf[starts[x // S] + x % S] (Section 4, the stride metadata of
    StridedRaggedShard; starts as dbuffer.strided_region_starts gives them)."""
    S = plan.S
    out = np.empty(plan.m * S, dtype=np.uint8)
    for k in range(plan.m):
        out[k * S:(k + 1) * S] = buf[starts[k]:starts[k] + S]
    return out


def dequant_unpack_strided(plan: Plan, buf: np.ndarray, starts, scales: np.ndarray, f32: bool = False) -> List[np.ndarray]:
    """dequant_unpack of one group's regions of a mesh-gathered code buffer: the reshuffle on
    materialise, with the group's own scale array."""
    logical = gather_strided_codes(plan, buf, starts)
    return dequant_unpack_f32(plan, logical, scales) if f32 else dequant_unpack(plan, logical, scales)


def dequant_unpack_f32(plan: Plan, codes: np.ndarray, scales: np.ndarray) -> List[np.ndarray]:
    """Per-parameter fp32 values from the gathered codes (m*S) and all scales."""
    out = []
    for spec, l, sb in zip(plan.specs, plan.offsets, plan.scale_bases()):
        if not spec.quantised:
            raise ValueError("dequant_unpack needs quantised tensors")
        out.append(dequantise_tensor_f32(codes[l:l + spec.e], scales[sb:sb + spec.num_blocks], spec))
    return out


def dequant_unpack(plan: Plan, codes: np.ndarray, scales: np.ndarray) -> List[np.ndarray]:
    """Per-parameter bf16 bits from the gathered codes (m*S) and all scales."""
    out = []
    for spec, l, sb in zip(plan.specs, plan.offsets, plan.scale_bases()):
        if not spec.quantised:
            raise ValueError("dequant_unpack needs quantised tensors")
        out.append(dequantise_tensor(codes[l:l + spec.e], scales[sb:sb + spec.num_blocks], spec))
    return out
