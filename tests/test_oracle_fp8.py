"""Pins for the FP8 oracle: the E4M3 format definition (hand-stated values), the library's
own float8_e4m3fn cast as an independent encoder/decoder, brute-force nearest search,
and the invariants block-wise quantisation must satisfy."""
import numpy as np
import pytest
import torch

from oracle import fp8 as F
from oracle import plan as P
from oracle.dbuffer import bf16_bits_to_f32, ragged_pack
from workloads import WORKLOADS, gen_params


def all_bf16_in_range():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    x = bf16_bits_to_f32(bits)
    keep = np.isfinite(x) & (np.abs(x) <= 448.0)
    return x[keep]


def test_decode_table_hand_values():
    tab = F.decode_table()
    assert tab[0x00] == 0.0 and tab[0x80] == 0.0 and np.signbit(tab[0x80])
    assert tab[0x01] == 2.0 ** -9            # smallest subnormal
    assert tab[0x07] == 0.875 * 2.0 ** -6    # largest subnormal
    assert tab[0x08] == 2.0 ** -6            # smallest normal
    assert tab[0x38] == 1.0
    assert tab[0x39] == 1.125
    assert tab[0x7E] == 448.0 and tab[0xFE] == -448.0
    assert np.isnan(tab[0x7F]) and np.isnan(tab[0xFF])
    pos = tab[:0x7F]
    assert np.all(np.diff(pos) > 0)


def test_decode_table_matches_library_format():
    codes = torch.arange(256, dtype=torch.int32).to(torch.uint8)
    lib = codes.view(torch.float8_e4m3fn).to(torch.float32).numpy()
    tab = F.decode_table()
    assert np.array_equal(np.isnan(lib), np.isnan(tab))
    ok = ~np.isnan(lib)
    assert np.array_equal(lib[ok].view(np.uint32), tab[ok].view(np.uint32))


def test_encode_hand_values():
    def enc(v):
        return int(F.encode_e4m3(np.array([v], dtype=np.float32))[0])
    assert enc(448.0) == 0x7E and enc(-448.0) == 0xFE
    assert enc(1.0) == 0x38
    assert enc(0.0) == 0x00 and enc(-0.0) == 0x80
    assert enc(2.0 ** -9) == 0x01
    assert enc(2.0 ** -10) == 0x00            # tie between 0 and 2^-9 -> even mantissa (0)
    assert enc(-(2.0 ** -10)) == 0x80         # ... keeping the sign
    assert enc(np.nextafter(np.float32(2.0 ** -10), np.float32(1))) == 0x01
    assert enc(3 * 2.0 ** -10) == 0x02        # tie between codes 1 and 2 -> 2
    assert enc(1.0625) == 0x38                # tie 1.0 / 1.125 -> even (1.0)
    assert enc(1.1875) == 0x3A                # tie 1.125 / 1.25 -> even (1.25)
    assert enc(432.0) == 0x7E                 # tie 416 / 448 -> 448 has the even mantissa (110)
    assert enc(447.9) == 0x7E
    assert enc(0.0146484375) == 0x08          # tie 0.875*2^-6 / 2^-6 -> normal 2^-6 (even)


def test_encode_equals_library_cast_on_every_bf16_value():
    x = all_bf16_in_range()
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(F.encode_e4m3(x), lib)


def test_encode_equals_library_cast_on_random_and_tie_fp32():
    rng = np.random.default_rng(0)
    x = np.concatenate([
        rng.uniform(-448, 448, 200000).astype(np.float32),
        (rng.standard_normal(200000) * 0.05).astype(np.float32),
        (rng.standard_normal(100000) * 2.0 ** -8).astype(np.float32),
    ])
    tab = F.decode_table()[:0x7F].astype(np.float64)
    mids = ((tab[:-1] + tab[1:]) / 2).astype(np.float32)      # all exactly representable
    near = np.concatenate([mids, np.nextafter(mids, np.float32(1000)), np.nextafter(mids, np.float32(-1))])
    x = np.concatenate([x, near, -near])
    lib = torch.from_numpy(x).to(torch.float8_e4m3fn).view(torch.uint8).numpy()
    assert np.array_equal(F.encode_e4m3(x), lib)


def test_encode_brute_force_nearest_with_ties_to_even():
    tab = [F.e4m3_value(c) for c in range(0x7F)]
    x = all_bf16_in_range()
    x = x[::7]
    got = F.encode_e4m3(x)
    for v, c in zip(x.tolist(), got.tolist()):
        a = abs(v)
        best = min(range(0x7F), key=lambda k: (abs(tab[k] - a), k & 1))
        assert (c & 0x7F) == best
        assert (c >> 7) == (1 if np.signbit(np.float32(v)) else 0)


def test_bf16_rounding_matches_library():
    rng = np.random.default_rng(1)
    x = np.concatenate([
        (rng.standard_normal(300000) * 0.02).astype(np.float32),
        rng.integers(0, 0x7F000000, 300000, dtype=np.int64).astype(np.uint32).view(np.float32),
        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38], dtype=np.float32),
    ])
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(F.f32_to_bf16_bits(x), lib)


def ref_quant_block_by_block(bits2d, bh, bw):
    """Independent restatement: python loops over blocks, library cast as the encoder."""
    R, C = bits2d.shape
    x = torch.from_numpy(bits2d.view(np.int16).copy()).view(torch.bfloat16).to(torch.float32)
    codes = torch.zeros((R, C), dtype=torch.uint8)
    scales = []
    for r0 in range(0, R, bh):
        row = []
        for c0 in range(0, C, bw):
            blk = x[r0:r0 + bh, c0:c0 + bw]
            amax = blk.abs().max()
            if amax == 0:
                row.append(0.0)
                continue
            scale = amax / torch.tensor(448.0, dtype=torch.float32)
            y = torch.clamp(blk / scale, -448.0, 448.0)
            codes[r0:r0 + bh, c0:c0 + bw] = y.to(torch.float8_e4m3fn).view(torch.uint8)
            row.append(float(scale))
        scales.append(row)
    return codes.numpy(), np.array(scales, dtype=np.float32)


@pytest.mark.parametrize("shape,bh,bw", [((257, 130), 128, 128), ((128, 128), 128, 128),
                                         ((300, 384), 128, 128), ((5, 300), 1, 128), ((1, 384), 1, 128),
                                         ((1, 100), 1, 128)])
def test_quantise_matrix_against_block_loop(shape, bh, bw):
    rng = np.random.default_rng(5)
    x = (rng.standard_normal(shape) * 0.02).astype(np.float32)
    x[0, 0] = 0.0
    bits = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    if shape == (300, 384):
        bits[128:256, 128:256] = 0            # an all-zero block
        bits[0:128, 0:128] = 0x8000           # a block of negative zeros
    c, s = F.quantise_matrix(bits, bh, bw)
    c2, s2 = ref_quant_block_by_block(bits, bh, bw)
    assert np.array_equal(s.view(np.uint32), s2.view(np.uint32))
    assert np.array_equal(c, c2)


def toy_plan():
    wl = WORKLOADS[1]
    specs = [P.TensorSpec(t.rows, t.cols, t.mode) for t in wl.tensors]
    return wl, P.make_plan(specs, wl.world, wl.align_bytes, wl.min_itemsize)


def test_every_nonzero_block_hits_the_largest_code():
    wl, pl = toy_plan()
    params = gen_params(wl, seed=1)
    db = ragged_pack(params, pl.offsets, pl.total)
    codes, scales = F.block_quant_all(pl, db)
    for spec, l, sb in zip(pl.specs, pl.offsets, pl.scale_bases()):
        R, C, bh, bw = F._as_2d(spec)
        c2 = codes[l:l + spec.e].reshape(R, C)
        nbc = -(-C // bw)
        for br in range(-(-R // bh)):
            for bc in range(nbc):
                blk = c2[br * bh:(br + 1) * bh, bc * bw:(bc + 1) * bw]
                assert scales[sb + br * nbc + bc] > 0
                assert np.any((blk & 0x7F) == 0x7E)            # the amax element maps to +-448
    # padding of the code buffer is 0x00
    mask = np.ones(pl.total, dtype=bool)
    for spec, l in zip(pl.specs, pl.offsets):
        mask[l:l + spec.e] = False
    assert np.all(codes[mask] == 0)


def test_shard_by_shard_equals_whole_tensor():
    # Section 2.1 / 4: with blocks whole on a rank, no scale metadata is exchanged
    wl, pl = toy_plan()
    db = ragged_pack(gen_params(wl, seed=2), pl.offsets, pl.total)
    codes, scales = F.block_quant_all(pl, db)
    for k in range(wl.world):
        c, s = F.block_quant_shard(pl, k, db[k * pl.S:(k + 1) * pl.S])
        lo, hi = pl.scale_range(k)
        assert np.array_equal(c, codes[k * pl.S:(k + 1) * pl.S])
        assert np.array_equal(s.view(np.uint32), scales[lo:hi].view(np.uint32))


def test_round_trip_error_bound():
    # |x^ - x| <= |x| (2^-4 + 2^-8) + scale 2^-10: half an E4M3 ulp (3 mantissa bits), the
    # subnormal half-spacing, and the final bf16 rounding
    wl, pl = toy_plan()
    params = gen_params(wl, seed=3)
    db = ragged_pack(params, pl.offsets, pl.total)
    codes, scales = F.block_quant_all(pl, db)
    outs = F.dequant_unpack(pl, codes, scales)
    for spec, sb, src, out in zip(pl.specs, pl.scale_bases(), params, outs):
        x = bf16_bits_to_f32(src).astype(np.float64)
        y = bf16_bits_to_f32(out).astype(np.float64)
        R, C, bh, bw = F._as_2d(spec)
        nbc = -(-C // bw)
        r, c = np.divmod(np.arange(spec.e), C)
        sc = scales[sb + (r // bh) * nbc + c // bw].astype(np.float64)
        assert np.all(np.abs(y - x) <= np.abs(x) * (2.0 ** -4 + 2.0 ** -8) + sc * 2.0 ** -10)
        assert np.array_equal(np.signbit(y[x != 0]), np.signbit(x[x != 0]))


def test_dequantise_against_library():
    wl, pl = toy_plan()
    db = ragged_pack(gen_params(wl, seed=4), pl.offsets, pl.total)
    codes, scales = F.block_quant_all(pl, db)
    outs = F.dequant_unpack(pl, codes, scales)
    for spec, l, sb, out in zip(pl.specs, pl.offsets, pl.scale_bases(), outs):
        R, C, bh, bw = F._as_2d(spec)
        nbc = -(-C // bw)
        v = torch.from_numpy(codes[l:l + spec.e].copy()).view(torch.float8_e4m3fn).to(torch.float32)
        r, c = np.divmod(np.arange(spec.e), C)
        sc = torch.from_numpy(scales[sb + (r // bh) * nbc + c // bw])
        lib = (v * sc).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
        assert np.array_equal(out, lib)


def test_dequantise_f32_against_library_and_exact_products():
    wl, pl = toy_plan()
    db = ragged_pack(gen_params(wl, seed=6), pl.offsets, pl.total)
    codes, scales = F.block_quant_all(pl, db)
    outs32 = F.dequant_unpack_f32(pl, codes, scales)
    outs16 = F.dequant_unpack(pl, codes, scales)
    tab = [F.e4m3_value(c) for c in range(256)]
    for spec, l, sb, o32, o16 in zip(pl.specs, pl.offsets, pl.scale_bases(), outs32, outs16):
        R, C, bh, bw = F._as_2d(spec)
        nbc = -(-C // bw)
        r, c = np.divmod(np.arange(spec.e), C)
        sidx = sb + (r // bh) * nbc + c // bw
        # library decode and multiply
        v = torch.from_numpy(codes[l:l + spec.e].copy()).view(torch.float8_e4m3fn).to(torch.float32)
        lib = (v * torch.from_numpy(scales[sidx])).numpy()
        assert o32.dtype == np.float32 and np.array_equal(o32.view(np.uint32), lib.view(np.uint32))
        # the product of a 4-bit and a 24-bit significand is exact in double: one rounding to fp32
        val = np.array([tab[k] for k in codes[l:l + spec.e]], dtype=np.float64)
        once = (val * scales[sidx].astype(np.float64)).astype(np.float32)
        assert np.array_equal(o32.view(np.uint32), once.view(np.uint32))
        # rounding it to bf16 gives the bf16 form
        assert np.array_equal(F.f32_to_bf16_bits(o32), o16)


# ---- fp32 inputs (the mean of the partials, quantised without passing through bf16) ----------

def ref_quant_f32_block_by_block(x2d, bh, bw):
    """Independent restatement for fp32 input: python loops over blocks, library cast as the
    encoder, library division."""
    x = torch.from_numpy(np.ascontiguousarray(x2d))
    R, C = x.shape
    codes = torch.zeros((R, C), dtype=torch.uint8)
    scales = []
    for r0 in range(0, R, bh):
        row = []
        for c0 in range(0, C, bw):
            blk = x[r0:r0 + bh, c0:c0 + bw]
            scale = blk.abs().max() / torch.tensor(448.0, dtype=torch.float32)
            if scale == 0:
                row.append(0.0)
                continue
            y = torch.clamp(blk / scale, -448.0, 448.0)
            codes[r0:r0 + bh, c0:c0 + bw] = y.to(torch.float8_e4m3fn).view(torch.uint8)
            row.append(float(scale))
        scales.append(row)
    return codes.numpy(), np.array(scales, dtype=np.float32)


@pytest.mark.parametrize("shape,bh,bw", [((257, 130), 128, 128), ((300, 384), 128, 128), ((5, 300), 1, 128)])
def test_quantise_f32_matrix_against_block_loop(shape, bh, bw):
    rng = np.random.default_rng(15)
    x = (rng.standard_normal(shape) * 1e-3).astype(np.float32)      # full fp32 mantissas
    x[0, 0] = 0.0
    if shape == (300, 384):
        x[128:256, 128:256] = 0.0                                   # an all-zero block
        x[0:128, 0:128] = -0.0
        x[256:300, 0:128] = np.float32(1e-44)                       # scale underflows: a zero block
        x[0:128, 256:384] *= np.float32(1e-36)                      # subnormal means, live block
    c, s = F.quantise_matrix_f32(x, bh, bw)
    c2, s2 = ref_quant_f32_block_by_block(x, bh, bw)
    assert np.array_equal(s.view(np.uint32), s2.view(np.uint32))
    assert np.array_equal(c, c2)
    if shape == (300, 384):
        assert s[2, 0] == 0 and np.all(c[256:300, 0:128] == 0)
        assert s[0, 2] > 0 and np.any(c[0:128, 256:384] == 0x7E)


def test_f32_and_bf16_quantisers_agree_on_bf16_values():
    rng = np.random.default_rng(16)
    bits = torch.from_numpy((rng.standard_normal((140, 260)) * 0.02).astype(np.float32)).to(
        torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    bits[:, 128:256] = 0x0001                                        # smallest bf16 subnormal: still live
    a = F.quantise_matrix(bits, 128, 128)
    b = F.quantise_matrix_f32(bf16_bits_to_f32(bits), 128, 128)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1].view(np.uint32), b[1].view(np.uint32))
    assert a[1][0, 1] > 0 and np.all(a[0][:128, 128:256] == 0x7E)


def test_fused_reduce_quantise_is_the_composition_and_stays_near_the_mean():
    from oracle.dbuffer import shard_reduce, shard_reduce_f32_ordered
    from workloads import gen_partial
    wl, pl = toy_plan()
    for k in (0, wl.world - 1):
        parts = np.stack([gen_partial(wl, 4, w, pl.S) for w in range(wl.world)])
        segs = pl.rank_segments(k)
        codes, scales, mean = F.reduce_quant_shard(pl, k, parts)
        assert np.array_equal(mean.view(np.uint32), shard_reduce_f32_ordered(parts, segs).view(np.uint32))
        lo, hi = pl.scale_range(k)
        assert scales.size == hi - lo
        # dequantised codes lie within half an E4M3 step of the float64 mean (plus the reduce's own bound)
        exact = shard_reduce(parts, segs).astype(np.float64)
        tab = F.decode_table().astype(np.float64)
        pos = 0
        for t, src_off, dst_off, n in segs:
            spec = pl.specs[t]
            sub = P.TensorSpec(n // spec.cols, spec.cols, spec.mode) if spec.cols else P.TensorSpec(n, 0, spec.mode)
            R, C, bh, bw = F._as_2d(sub)
            nbc = -(-C // bw)
            r, c = np.divmod(np.arange(n), C)
            sc = scales[pos + (r // bh) * nbc + c // bw].astype(np.float64)
            pos += sub.num_blocks
            back = tab[codes[dst_off:dst_off + n]] * sc
            x = exact[dst_off:dst_off + n]
            assert np.all(np.abs(back - x) <= np.abs(x) * 2.0 ** -4 + sc * 2.0 ** -10 + 1e-9)
        assert pos == scales.size
        pay = np.zeros(pl.S, dtype=bool)
        for _, _, d, n in segs:
            pay[d:d + n] = True
        assert np.all(codes[~pay] == 0) and np.all(mean[~pay] == 0)


def test_fused_reduce_quantise_against_the_definition_alone():
    """The fused function's scales and codes held against the float64 mean with no summation order
    assumed (the check the GPU tests apply at full size), on the toy unit and on a unit with row
    blocks, a 1-D tensor and ragged edges; and the check does catch a planted mistake (a dropped
    partial, a sum in place of the mean, a scale from the wrong block)."""
    from fused_check import order_free_fused_check
    from workloads import gen_partial, normal_bf16
    wl, pl = toy_plan()
    ragged = [P.TensorSpec(300, 384, P.BLOCK_128x128), P.TensorSpec(1000, 0, P.BLOCK_1x128),
              P.TensorSpec(257, 136, P.BLOCK_128x128), P.TensorSpec(64, 200, P.BLOCK_1x128)]
    pr = P.make_plan(ragged, 3)
    for plan, W, draw in ((pl, wl.world, lambda w, S: gen_partial(wl, 4, w, S)),
                          (pr, 3, lambda w, S: normal_bf16(8, 3, 1, w, S, 1e-3))):
        for k in range(plan.m):
            parts = np.stack([draw(w, plan.S) for w in range(W)])
            codes, scales, _ = F.reduce_quant_shard(plan, k, parts)
            get = lambda a, b: np.ascontiguousarray(parts[:, a:b])
            n = order_free_fused_check(plan, plan.specs, k, get, codes, scales, "oracle")
            assert n == sum(s[3] for s in plan.rank_segments(k))
            if n == 0:
                continue
            # planted mistakes must be caught
            dropped = parts.copy()
            dropped[W - 1] = 0
            c2, s2, _ = F.reduce_quant_shard(plan, k, dropped)
            with pytest.raises(AssertionError):
                order_free_fused_check(plan, plan.specs, k, get, c2, s2, "dropped partial")
            with pytest.raises(AssertionError):
                order_free_fused_check(plan, plan.specs, k, get, codes, scales * np.float32(W), "sum, not mean")
            if scales.size > 2:
                with pytest.raises(AssertionError):
                    order_free_fused_check(plan, plan.specs, k, get, codes, np.roll(scales, 1), "scales shifted")


def test_strided_dequant_unpack_against_reshape_and_per_element_gather():
    """FP8 codes gathered over a (m x groups) mesh, FSDP rank outermost: one group's logical code
    buffer is a strided slice (numpy reshape as the independent formulation), its unpack is the
    plain dequant_unpack of that slice, and single elements follow the address rule by hand."""
    from oracle.dbuffer import strided_region_starts
    wl, pl = toy_plan()
    m, S, groups = pl.m, pl.S, 3
    rng = np.random.default_rng(12)
    gathered = rng.integers(0, 0x7F, size=m * groups * S, dtype=np.uint8) | (
        rng.integers(0, 2, size=m * groups * S, dtype=np.uint8) << 7)           # any code but NaN
    nb = pl.scale_bases()[-1]
    tab = F.decode_table()
    for grp in range(groups):
        scales = (rng.random(nb).astype(np.float32) + np.float32(0.5)) * np.float32(1e-3)
        starts = strided_region_starts(m, S, groups, grp)
        logical = gathered.reshape(m, groups, S)[:, grp, :].reshape(-1)
        assert np.array_equal(F.gather_strided_codes(pl, gathered, starts), logical)
        for f32 in (False, True):
            got = F.dequant_unpack_strided(pl, gathered, starts, scales, f32=f32)
            want = F.dequant_unpack_f32(pl, logical, scales) if f32 else F.dequant_unpack(pl, logical, scales)
            for a, b in zip(got, want):
                assert np.array_equal(a, b)
        # by hand on tensor 0 (256 x 384, 128x128 tiles): element (row, col) of the fp32 form
        got = F.dequant_unpack_strided(pl, gathered, starts, scales, f32=True)
        l, C = pl.offsets[0], 384
        for row, col in ((0, 0), (127, 383), (128, 5), (255, 200)):
            x = l + row * C + col
            code = gathered[((x // S) * groups + grp) * S + x % S]
            blk = pl.scale_bases()[0] + (row // 128) * 3 + col // 128
            assert got[0][row * C + col] == tab[code] * scales[blk]
