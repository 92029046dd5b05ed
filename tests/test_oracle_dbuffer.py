"""Pins for the DBuffer oracle: per-element brute force for pack / unpack, exact
arithmetic (fractions / fsum) and special cases for shard_reduce."""
import math

import numpy as np

from oracle import dbuffer as D
from oracle import plan as P
from workloads import WORKLOADS, gen_params, gen_partial


def toy():
    wl = WORKLOADS[1]
    specs = [P.TensorSpec(t.rows, t.cols, t.mode) for t in wl.tensors]
    return wl, P.make_plan(specs, wl.world, wl.align_bytes, wl.min_itemsize)


def test_pack_per_element_scatter_and_zero_padding():
    wl, pl = toy()
    params = gen_params(wl, seed=1)
    db = D.ragged_pack(params, pl.offsets, pl.total)
    want = [0] * pl.total
    for src, l in zip(params, pl.offsets):
        for i, v in enumerate(src.tolist()):
            want[l + i] = v
    assert db.tolist() == want
    assert db.size == wl.world * pl.S
    inside = np.zeros(pl.total, dtype=bool)
    for s, l in zip(pl.specs, pl.offsets):
        inside[l:l + s.e] = True
    assert np.all(db[~inside] == 0)


def test_unpack_inverts_pack():
    wl, pl = toy()
    params = gen_params(wl, seed=2)
    db = D.ragged_pack(params, pl.offsets, pl.total)
    outs = D.unpack_bf16(db, pl.offsets, [s.e for s in pl.specs])
    for a, b in zip(params, outs):
        assert np.array_equal(a, b)


def test_bf16_widening_is_bit_placement():
    bits = np.array([0x3F80, 0xBF80, 0x0001, 0x7F7F, 0x0000, 0x8000], dtype=np.uint16)
    f = D.bf16_bits_to_f32(bits)
    assert f[0] == 1.0 and f[1] == -1.0 and f[2] == 2.0 ** -133
    assert f[3] == (2 - 2.0 ** -7) * 2.0 ** 127
    assert f[4] == 0 and np.signbit(f[5])


def test_reduce_exact_rational_on_sample():
    wl, pl = toy()
    k = 1
    segs = pl.rank_segments(k)
    parts = np.stack([gen_partial(wl, 3, w, pl.S) for w in range(wl.world)])
    out = D.shard_reduce(parts, segs)
    payload = np.zeros(pl.S, dtype=bool)
    for _, _, d, n in segs:
        payload[d:d + n] = True
    assert np.all(out[~payload] == 0)
    assert (~payload).any()
    idx = np.flatnonzero(payload)[::97]
    for i in idx.tolist():
        vals = [float(D.bf16_bits_to_f32(parts[w, i:i + 1])[0]) for w in range(wl.world)]
        exact = math.fsum(vals) / wl.world            # fsum is exact, one rounding in the division
        assert out[i] == np.float32(exact)


def test_reduce_special_cases():
    S = 64
    segs = [(0, 0, 0, 40), (1, 0, 48, 16)]
    one = gen_partial(WORKLOADS[1], 4, 0, S).reshape(1, S)
    out = D.shard_reduce(one, segs)
    widened = D.bf16_bits_to_f32(one[0])
    assert np.array_equal(out[:40], widened[:40]) and np.array_equal(out[48:], widened[48:])
    assert np.all(out[40:48] == 0)                    # padding stays 0 whatever the partials hold
    same = np.repeat(one, 8, axis=0)                  # equal partials, W a power of two
    assert np.array_equal(D.shard_reduce(same, segs), out)
    neg = same.copy()
    neg[1::2] ^= 0x8000                               # alternate signs cancel exactly
    assert np.all(D.shard_reduce(neg, segs) == 0)
    # the mean, not the sum: W = 4 partials of 1.0, 2.0, 3.0, 6.0 -> 3.0
    vals = np.array([[0x3F80], [0x4000], [0x4040], [0x40C0]], dtype=np.uint16)
    assert D.shard_reduce(vals, [(0, 0, 0, 1)])[0] == 3.0
    assert D.shard_reduce_abs_sum(vals)[0] == 12.0


def test_ordered_fp32_reduce_stays_within_the_stated_tolerance_and_follows_its_order():
    from fractions import Fraction
    wl, pl = toy()
    for W in (1, 3, 8, 13, 64):
        S = 4096
        parts = np.stack([gen_partial(wl, 5, w, S) for w in range(W)])
        segs = [(0, 0, 0, 1000), (1, 0, 1024, 3000)]
        exact = D.shard_reduce(parts, segs)
        got = D.shard_reduce_f32_ordered(parts, segs)
        bound = 1e-5 * D.shard_reduce_abs_sum(parts)
        assert np.all(np.abs(got.astype(np.float64) - exact.astype(np.float64)) <= bound)
        assert np.all(got[1000:1024] == 0) and np.all(got[4024:] == 0)
        # the order, element by element on a sample, with exact rationals rounded to fp32 at every step
        def rn(q):
            return Fraction(float(np.float32(float(q)))) if q != 0 else q   # double holds the exact sum of two fp32
        for i in (0, 17, 999, 1024, 2500, 4023):
            sums = [Fraction(0)] * 8
            for w in range(W):
                x = Fraction(float(D.bf16_bits_to_f32(parts[w, i:i + 1])[0]))
                sums[w % 8] = rn(sums[w % 8] + x)
            tot = rn(rn(rn(sums[0] + sums[1]) + rn(sums[2] + sums[3])) + rn(rn(sums[4] + sums[5]) + rn(sums[6] + sums[7])))
            inv = Fraction(float(np.float32(1.0) / np.float32(W)))
            want = np.float32(float(tot * inv))
            assert got[i] == want, (W, i)
    # W <= 8 with equal partials and W a power of two: the value itself
    same = np.repeat(parts[:1], 8, axis=0)
    assert np.array_equal(D.shard_reduce_f32_ordered(same, [(0, 0, 0, S)]), D.bf16_bits_to_f32(same[0]))


def test_strided_regions_against_reshape_and_per_element_gather():
    """A buffer gathered over a (m x groups) mesh, FSDP rank outermost: the logical buffer of one
    group is a strided slice; unpacking it equals plain unpack of that slice (numpy reshape as the
    independent formulation) and a per-element gather; pack is the inverse and leaves other
    groups' regions alone."""
    wl, pl = toy()
    m, S, groups = pl.m, pl.S, 3
    sizes = [s.e for s in pl.specs]
    rng = np.random.default_rng(9)
    gathered = rng.integers(0, 1 << 16, size=m * groups * S, dtype=np.uint16)
    for grp in range(groups):
        starts = D.strided_region_starts(m, S, groups, grp)
        assert starts == [(k * groups + grp) * S for k in range(m)]
        logical = gathered.reshape(m, groups, S)[:, grp, :].reshape(-1)
        want = D.unpack_bf16(logical, pl.offsets, sizes)
        got = D.unpack_bf16_strided(gathered, pl.offsets, sizes, S, starts)
        for a, b in zip(got, want):
            assert np.array_equal(a, b)
        t, l = 3, pl.offsets[3]
        for i in (0, 1, sizes[t] // 2, sizes[t] - 1):
            x = l + i
            assert got[t][i] == gathered[((x // S) * groups + grp) * S + x % S]
        # pack back: the group's regions hold the packed unit, the others are untouched
        packed = D.ragged_pack_strided(gathered, got, pl.offsets, S, starts)
        back = packed.reshape(m, groups, S)
        assert np.array_equal(back[:, grp, :].reshape(-1), D.ragged_pack(got, pl.offsets, pl.total))
        for other in range(groups):
            if other != grp:
                assert np.array_equal(back[:, other, :], gathered.reshape(m, groups, S)[:, other, :])
    # one group is the plain layout
    starts = D.strided_region_starts(m, S, 1, 0)
    flat = gathered[:pl.total]
    for a, b in zip(D.unpack_bf16_strided(flat, pl.offsets, sizes, S, starts), D.unpack_bf16(flat, pl.offsets, sizes)):
        assert np.array_equal(a, b)
