"""Oracle for the block-wise 8-bit optimiser state on a ragged shard and the Adam step on it.
TEST INFRASTRUCTURE ONLY - never imported by the product.

Section 6.3 ("8-bit Adam optimizer"): the two gradient statistics of Adam are kept as
block-wise INT8 with 32x32 blocks; matrix parameters get 32-row sharding granularity, so
every block is whole on one device and each device (re)quantises its local shard with no
communication.  The paper fixes the block shape and nothing else; the reading taken:

  state blocks   2-D tensor whose granularity is a multiple of 32 rows (32x32 or 128x128 mode):
                 32x32 tiles, edge tiles partial.  1-D tensor of granularity 128 (32x32 or
                 1x128 mode): runs of 128 elements.  2-D tensor of one-row granularity (1x128
                 mode): runs of 128 along each row, the last run of a row short - the finest
                 blocks that are whole on a rank there.  Other tensors have none.  A rank's
                 blocks are contiguous in the flat per-unit block order (tensor-major in
                 buffer order, then block row, then block column).
  code maps      linear absmax (the non-linear code book of the cited 8-bit optimiser paper
                 is not given):  first moment  m: absmax a, step s = a / 127, code = rint(m / s)
                 in [-127, 127];  second moment v >= 0: absmax a, step s = a / 255,
                 code = rint(v / s) in [0, 255].  rint = nearest, ties to even.  a == 0: codes 0.
                 value(code) = code * s.
  one step       all in fp32, every operation rounded on its own, in this order:
                   m_old = code_m * (a_m / 127)          v_old = code_v * (a_v / 255)
                   m = beta1 * m_old + (1 - beta1) * g
                   v = beta2 * v_old + (1 - beta2) * (g * g)
                   w = w * (1 - lr * weight_decay)                    (decoupled decay)
                   w = w - (lr / bc1) * ( m / ( sqrt(v) / sqrt(bc2) + eps ) )
                   param = bf16(w), nearest even
                 with bc_i = 1 - beta_i^step.  The seven constants beta_i, (1 - beta_i), eps,
                 lr / bc1, sqrt(bc2) and (1 - lr * weight_decay) are evaluated in double
                 precision from the hyper-parameters and rounded once to fp32.
                 Then m and v are quantised again block by block.
  buffers        g, w: fp32 at the element offsets of the rank's region; codes likewise
                 (int8 / uint8); padding positions are never read or written.
"""
from __future__ import annotations

from dataclasses import dataclass
from math import sqrt
from typing import List, Tuple

import numpy as np

from .plan import BLOCK_128x128, BLOCK_1x128, BLOCK_32x32, Plan, TensorSpec, ceil_div

F = np.float32


def state_runs(spec: TensorSpec) -> bool:
    """True where the state blocks are runs of 128 along each row, False where they are tiles."""
    if spec.cols == 0 and spec.mode in (BLOCK_1x128, BLOCK_32x32):
        return True
    if spec.cols > 0 and spec.mode == BLOCK_1x128:
        return True
    if spec.cols > 0 and spec.mode in (BLOCK_128x128, BLOCK_32x32):
        return False
    raise ValueError("no 8-bit state blocks for this sharding granularity")


def state_grid(spec: TensorSpec) -> Tuple[int, int]:
    """(rows of state blocks, state blocks per row of blocks) of one tensor."""
    if state_runs(spec):
        return (ceil_div(spec.rows, 128), 1) if spec.cols == 0 else (spec.rows, ceil_div(spec.cols, 128))
    return ceil_div(spec.rows, 32), ceil_div(spec.cols, 32)


def state_bases(plan: Plan) -> List[int]:
    """First state block of every tensor (indexed like plan.specs), then the total."""
    out, acc = [0] * (len(plan.specs) + 1), 0
    for t in plan.buffer_order():
        out[t] = acc
        nbr, nbc = state_grid(plan.specs[t])
        acc += nbr * nbc
    out[-1] = acc
    return out


def state_range(plan: Plan, k: int) -> Tuple[int, int]:
    """[lo, hi): the state blocks rank k owns."""
    def before(x):
        n = 0
        for s, l in zip(plan.specs, plan.offsets):
            nbr, nbc = state_grid(s)
            have = min(max(x - l, 0), s.e)          # elements of the tensor in front of x
            if s.cols == 0:
                n += ceil_div(have, 128)
            else:
                assert have % s.cols == 0           # rank boundaries fall between rows
                rows = have // s.cols
                n += rows * nbc if state_runs(s) else ceil_div(rows, 32) * nbc
        return n
    return before(k * plan.S), before((k + 1) * plan.S)


def _blocks(R: int, C: int, one_d: bool):
    """Yields (block index, row slice, col slice) of the state blocks of an (R, C) matrix:
    runs of 128 along each row (one_d; a 1-D tensor is the matrix (1, n)), else 32x32 tiles."""
    if one_d:
        per_row = ceil_div(C, 128)
        for r in range(R):
            for b in range(per_row):
                yield r * per_row + b, slice(r, r + 1), slice(b * 128, min(C, (b + 1) * 128))
        return
    nbc = ceil_div(C, 32)
    for br in range(ceil_div(R, 32)):
        for bc in range(nbc):
            yield br * nbc + bc, slice(br * 32, min(R, (br + 1) * 32)), slice(bc * 32, min(C, (bc + 1) * 32))


def quantise_state(x: np.ndarray, one_d: bool, signed: bool) -> Tuple[np.ndarray, np.ndarray]:
    """x: (R, C) fp32.  Returns codes (R, C) int16 (holding int8 / uint8 values) and absmax per block."""
    R, C = x.shape
    levels = F(127.0) if signed else F(255.0)
    codes = np.zeros((R, C), dtype=np.int16)
    nblk = R * ceil_div(C, 128) if one_d else ceil_div(R, 32) * ceil_div(C, 32)
    amax = np.zeros(nblk, dtype=np.float32)
    for b, rs, cs in _blocks(R, C, one_d):
        blk = x[rs, cs].astype(np.float32)
        a = F(np.max(np.abs(blk))) if signed else F(np.max(blk))
        amax[b] = a
        if a == 0:
            continue
        step = a / levels                                    # fp32 / fp32
        q = np.rint(blk / step)                              # fp32 / fp32, ties to even
        lo = -127.0 if signed else 0.0
        codes[rs, cs] = np.clip(q, lo, float(levels)).astype(np.int16)
    return codes, amax


def dequantise_state(codes: np.ndarray, amax: np.ndarray, one_d: bool, signed: bool) -> np.ndarray:
    R, C = codes.shape
    levels = F(127.0) if signed else F(255.0)
    out = np.zeros((R, C), dtype=np.float32)
    for b, rs, cs in _blocks(R, C, one_d):
        step = F(amax[b]) / levels
        out[rs, cs] = codes[rs, cs].astype(np.float32) * step
    return out


def _segments(plan: Plan, k: int):
    """(dst_off, n, R, C, runs, blocks) of every segment of rank k's region: a segment is a run of
    whole granules of one tensor, i.e. a matrix of whole state blocks."""
    out = []
    for t, src_off, dst_off, n in plan.rank_segments(k):
        spec = plan.specs[t]
        runs = state_runs(spec)
        if spec.cols == 0:
            assert src_off % 128 == 0
            R, C, nblk = 1, n, ceil_div(n, 128)
        else:
            assert n % spec.cols == 0 and src_off % (spec.cols if runs else 32 * spec.cols) == 0
            R, C = n // spec.cols, spec.cols
            nblk = R * ceil_div(C, 128) if runs else ceil_div(R, 32) * ceil_div(C, 32)
        out.append((dst_off, n, R, C, runs, nblk))
    return out


def quantise_shard(plan: Plan, k: int, x: np.ndarray, codes: np.ndarray, signed: bool):
    """The codec on its own over rank k's region: x (S,) fp32 -> (codes, absmax slice).
    `codes` gives the array's padding contents (they are kept); int8 when signed, else uint8."""
    codes = codes.copy()
    amax = []
    for dst_off, n, R, C, runs, _ in _segments(plan, k):
        c, a = quantise_state(x[dst_off:dst_off + n].reshape(R, C), runs, signed)
        codes[dst_off:dst_off + n] = c.reshape(-1).astype(codes.dtype)
        amax.append(a)
    return codes, (np.concatenate(amax).astype(np.float32) if amax else np.zeros(0, np.float32))


def dequantise_shard(plan: Plan, k: int, codes: np.ndarray, amax: np.ndarray, out: np.ndarray, signed: bool):
    """Inverse map over rank k's region: value(code) = code * (absmax / levels); `out` gives the
    fp32 array's padding contents (they are kept)."""
    out = out.copy()
    cursor = 0
    for dst_off, n, R, C, runs, nblk in _segments(plan, k):
        c = codes[dst_off:dst_off + n].astype(np.int16).reshape(R, C)
        out[dst_off:dst_off + n] = dequantise_state(c, amax[cursor:cursor + nblk], runs, signed).reshape(-1)
        cursor += nblk
    assert cursor == amax.size
    return out


@dataclass
class Hyper:
    lr: float
    beta1: float
    beta2: float
    eps: float
    weight_decay: float
    step: int

    def derived(self):
        """The fp32 constants of a step: each is evaluated in double precision from the
        hyper-parameters as given and rounded once to fp32."""
        bc1 = 1.0 - self.beta1 ** self.step
        bc2 = 1.0 - self.beta2 ** self.step
        return dict(b1=F(self.beta1), b2=F(self.beta2), omb1=F(1.0 - self.beta1), omb2=F(1.0 - self.beta2),
                    eps=F(self.eps), step_size=F(self.lr / bc1), bc2s=F(sqrt(bc2)),
                    decay=F(1.0 - self.lr * self.weight_decay))


def adam_update(g: np.ndarray, w: np.ndarray, m_old: np.ndarray, v_old: np.ndarray, h: Hyper):
    """The fp32 update of the docstring on arrays of one shape: returns (m, v, w_new)."""
    d = h.derived()
    g = g.astype(np.float32)
    m = d["b1"] * m_old + d["omb1"] * g
    v = d["b2"] * v_old + d["omb2"] * (g * g)
    w1 = w.astype(np.float32) * d["decay"]
    denom = np.sqrt(v) / d["bc2s"] + d["eps"]
    w2 = w1 - d["step_size"] * (m / denom)
    return m.astype(np.float32), v.astype(np.float32), w2.astype(np.float32)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    keep = (u >> np.uint64(16)) & np.uint64(1)
    return ((u + np.uint64(0x7FFF) + keep) >> np.uint64(16)).astype(np.uint16)


def adam8_step_matrix(g, w, mc, vc, am, av, one_d: bool, h: Hyper):
    """One step on an (R, C) matrix that holds whole state blocks.
    Returns (w_new fp32, param bf16 bits, mc_new int16, vc_new int16, am_new, av_new)."""
    m_old = dequantise_state(mc, am, one_d, True)
    v_old = dequantise_state(vc, av, one_d, False)
    m, v, w_new = adam_update(g, w, m_old, v_old, h)
    mc_new, am_new = quantise_state(m, one_d, True)
    vc_new, av_new = quantise_state(v, one_d, False)
    return w_new, f32_to_bf16_bits(w_new), mc_new, vc_new, am_new, av_new


def adam8_step_shard(plan: Plan, k: int, g, w, param_bits, mc, vc, am, av, h: Hyper):
    """One step on rank k's region from nothing but that region.

    g, w: (S,) fp32; param_bits: (S,) uint16; mc: (S,) int8; vc: (S,) uint8;
    am, av: the rank's slices of the two absmax arrays.  Returns new copies of
    (w, param_bits, mc, vc, am, av); padding positions keep their input values."""
    w, param_bits, mc, vc = w.copy(), param_bits.copy(), mc.copy(), vc.copy()
    am_out, av_out = [], []
    cursor = 0
    for t, src_off, dst_off, n in plan.rank_segments(k):
        spec = plan.specs[t]
        one_d = state_runs(spec)
        if spec.cols == 0:
            assert src_off % 128 == 0
            R, C = 1, n
            nblk = ceil_div(n, 128)
        elif one_d:
            assert src_off % spec.cols == 0 and n % spec.cols == 0
            R, C = n // spec.cols, spec.cols
            nblk = R * ceil_div(C, 128)
        else:
            assert src_off % (32 * spec.cols) == 0 and n % spec.cols == 0
            R, C = n // spec.cols, spec.cols
            nblk = ceil_div(R, 32) * ceil_div(C, 32)
        sl = slice(dst_off, dst_off + n)
        res = adam8_step_matrix(g[sl].reshape(R, C), w[sl].reshape(R, C),
                                mc[sl].astype(np.int16).reshape(R, C), vc[sl].astype(np.int16).reshape(R, C),
                                am[cursor:cursor + nblk], av[cursor:cursor + nblk], one_d, h)
        w[sl] = res[0].reshape(-1)
        param_bits[sl] = res[1].reshape(-1)
        mc[sl] = res[2].reshape(-1).astype(np.int8)
        vc[sl] = res[3].reshape(-1).astype(np.uint8)
        am_out.append(res[4])
        av_out.append(res[5])
        cursor += nblk
    assert cursor == am.size == av.size
    cat = lambda xs: np.concatenate(xs).astype(np.float32) if xs else np.zeros(0, dtype=np.float32)
    return w, param_bits, mc, vc, cat(am_out), cat(av_out)
