"""The fused reduce + quantise held against the plain definition, with no summation order assumed
(shared by the CPU pin of the oracle's fused function and the GPU parity tests)."""
import numpy as np

from oracle import dbuffer as OD
from oracle import fp8 as OF
from oracle import plan as OP

REDUCE_TOL = 1e-5


def order_free_fused_check(plan, specs, rank, get_parts, codes, scales, label, reducer=OD, budget=1 << 27):
    """rs_reduce_quantize against the plain definition, with no summation order assumed: the mean
    is the float64 mean (to within the benchmark spec's 1e-5 * sum|x| per element); every scale is the
    block maximum of that mean / 448 to within that tolerance / 448; every code, decoded and
    multiplied by its scale, is the mean to within half an E4M3 step at that magnitude plus the
    tolerance.  get_parts(a, b): the (W, b - a) bf16 bits of region columns [a, b) on the host;
    codes (S), scales (the rank's slice): the results under test; plan / specs: the oracle's
    plan and tensor specs; reducer: the module whose float64 shard_reduce and shard_reduce_abs_sum
    are used (the numpy oracle, or its plain-C statement on large inputs).  The region is walked in pieces of
    whole rows of blocks, at most `budget` partial elements at a time.  Returns the elements checked."""
    table = OF.decode_table().astype(np.float64)
    sb = plan.scale_bases()
    lo, _ = plan.scale_range(rank)
    W = plan.m
    checked = 0
    for t, src_off, dst_off, n in plan.rank_segments(rank):
        spec = specs[t]
        tile = spec.mode == OP.BLOCK_128x128
        if spec.cols:
            C, bh, nbc = spec.cols, (128 if tile else 1), -(-spec.cols // 128)
            g = bh * C                       # one row of blocks
        else:
            C, bh, nbc, g = 128, 1, 1, 128   # a 1-D tensor as rows of 128, the last one short
        assert src_off % g == 0
        piece = max(g, budget // W // g * g)
        for a in range(0, n, piece):
            m_len = min(piece, n - a)
            parts = get_parts(dst_off + a, dst_off + a + m_len)
            seg = [(0, 0, 0, m_len)]
            mean = reducer.shard_reduce(parts, seg).astype(np.float64)
            tol = REDUCE_TOL * reducer.shard_reduce_abs_sum(parts)
            rows = -(-m_len // C)
            nbr = -(-rows // bh)
            first = sb[t] + (src_off + a) // g * nbc - lo
            sc = scales[first:first + nbr * nbc].astype(np.float64).reshape(nbr, nbc)
            full = nbr * bh * nbc * 128

            def grid(x):                     # (nbr, bh, nbc, 128) view, zero where nothing exists
                x2 = np.zeros((nbr * bh, nbc * 128), dtype=np.float64)
                flat = np.zeros(rows * C, dtype=np.float64)
                flat[:m_len] = x
                x2[:rows, :C] = flat.reshape(rows, C)
                return x2.reshape(nbr, bh, nbc, 128)
            amax = np.abs(grid(mean)).max(axis=(1, 3))
            tmax = grid(tol).max(axis=(1, 3))
            assert np.all(np.abs(sc - amax / 448.0) <= tmax / 448.0 + amax * 2.0 ** -22), f"{label}: scales of tensor {t}"
            per_elem = np.broadcast_to(sc[:, None, :, None], (nbr, bh, nbc, 128)).reshape(nbr * bh, nbc * 128)
            per_elem = per_elem[:rows, :C].reshape(-1)[:m_len]
            dec = table[codes[dst_off + a:dst_off + a + m_len]]
            value = dec * per_elem
            bound = per_elem * np.maximum(np.abs(dec) / 16.0, 2.0 ** -10) + tol * 1.125 + np.abs(mean) * 2.0 ** -20
            assert np.all(np.abs(value - mean) <= bound), f"{label}: codes of tensor {t}"
            assert full >= m_len
            checked += m_len
    return checked
