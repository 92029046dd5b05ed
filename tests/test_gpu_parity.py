"""GPU parity: every kernel of the HIP library against the CPU oracle, element by element, on
the same seeded inputs, through the C ABI.  Bit-exact for pack / unpack / FP8 codes / scales;
|err| <= 1e-5 * sum_w |x_w| per element for shard_reduce against the float64 definition, and
bit for bit against the fp32 sum in the stated order."""
import numpy as np
import pytest
import torch

from oracle import dbuffer as OD
from oracle import fp8 as OF
from paper_2602_22437_amd import binding as B
from workloads import (MODE_128x128, MODE_1x128, MODE_WHOLE, WORKLOADS, gen_params, gen_partial,
                       normal_bf16, uniform_bits)

from gpu_util import Unit, bits_of, say, to_dev_bf16

pytestmark = pytest.mark.gpu

REDUCE_TOL = 1e-5


def run_pack(u: Unit, params):
    dev = [to_dev_bf16(p) for p in params]
    dbuf = torch.full((u.total,), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)  # garbage
    B.rs_pack(u.plan, u.table(dev), dbuf)
    torch.cuda.synchronize()
    return dbuf


def check_pack_unpack(u: Unit, params, label):
    say(f"pack {label}: S={u.S} total={u.total}")
    dbuf = run_pack(u, params)
    want = OD.ragged_pack(params, u.oracle.offsets, u.total)
    assert np.array_equal(bits_of(dbuf), want), f"ragged_pack differs ({label})"
    say(f"unpack_bf16 {label}")
    outs = [torch.full((p.size,), 0x7FC0, dtype=torch.int16, device="cuda").view(torch.bfloat16) for p in params]
    B.rs_unpack_bf16(u.plan, dbuf, u.table(outs))
    torch.cuda.synchronize()
    for i, (o, p) in enumerate(zip(outs, params)):
        assert np.array_equal(bits_of(o), p), f"unpack_bf16 tensor {i} differs ({label})"
    return dbuf, want


def check_reduce(u: Unit, rank, partial_bits, label, poison_padding=True):
    """partial_bits: (W, S) uint16.  Padding columns may hold anything: the result is 0 there."""
    W, S = partial_bits.shape
    segs = u.oracle.rank_segments(rank)
    if poison_padding:
        pay = np.zeros(S, dtype=bool)
        for _, _, d, n in segs:
            pay[d:d + n] = True
        partial_bits = partial_bits.copy()
        partial_bits[:, ~pay] = 0x4300          # 128.0 where the kernel must not look
    say(f"reduce {label}: rank={rank} W={W} S={S}")
    dev = to_dev_bf16(partial_bits.reshape(-1))
    out = torch.full((S,), float("nan"), dtype=torch.float32, device="cuda")
    if W == u.world:
        B.rs_reduce(u.plan, rank, dev, S, out)
    else:
        B.rs_reduce_rows(u.plan, rank, dev, W, S, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    want = OD.shard_reduce(partial_bits, segs)
    bound = REDUCE_TOL * OD.shard_reduce_abs_sum(partial_bits)
    err = np.abs(got.astype(np.float64) - want.astype(np.float64))
    pay = np.zeros(S, dtype=bool)
    for _, _, d, n in segs:
        pay[d:d + n] = True
    assert np.all(got[~pay] == 0), f"reduce padding not zero ({label})"
    assert not np.any(np.isnan(got))
    assert np.all(err[pay] <= bound[pay]), f"reduce error above bound ({label}): {err.max()}"
    # and bit for bit the fp32 sum in the library's stated order
    ordered = OD.shard_reduce_f32_ordered(partial_bits, segs)
    assert np.array_equal(got.view(np.uint32), ordered.view(np.uint32)), f"reduce order differs ({label})"
    return got


def check_reduce_quant(u: Unit, rank, partial_bits, label):
    """The fused reduce + quantise against the oracle's composition, with and without the fp32
    mean written out; the mean must also equal rs_reduce bit for bit."""
    W, S = partial_bits.shape
    say(f"reduce_quantize {label}: rank={rank} W={W} S={S}")
    want_c, want_s, want_mean = OF.reduce_quant_shard(u.oracle, rank, partial_bits)
    lo, hi = u.oracle.scale_range(rank)
    dev = to_dev_bf16(partial_bits.reshape(-1))
    for with_mean in (False, True):
        codes = torch.full((S,), 0xEE, dtype=torch.uint8, device="cuda")
        scales = torch.full((max(hi - lo, 1),), float("nan"), dtype=torch.float32, device="cuda")
        mean = torch.full((S,), float("nan"), dtype=torch.float32, device="cuda") if with_mean else None
        B.rs_reduce_quantize(u.plan, rank, dev, S, codes, scales, mean)
        torch.cuda.synchronize()
        got_s = scales.cpu().numpy()[:hi - lo]
        assert np.array_equal(got_s.view(np.uint32), want_s.view(np.uint32)), f"fused scales differ ({label})"
        got_c = codes.cpu().numpy()
        if not np.array_equal(got_c, want_c):
            bad = np.flatnonzero(got_c != want_c)
            raise AssertionError(f"fused codes differ ({label}) at {bad[:8]}: got {got_c[bad[:8]]} "
                                 f"want {want_c[bad[:8]]}")
        if with_mean:
            assert np.array_equal(mean.cpu().numpy().view(np.uint32), want_mean.view(np.uint32)), \
                f"fused mean differs ({label})"
            out = torch.empty(S, dtype=torch.float32, device="cuda")
            B.rs_reduce(u.plan, rank, dev, S, out)
            torch.cuda.synchronize()
            assert torch.equal(out.view(torch.int32), mean.view(torch.int32)), f"fused mean != rs_reduce ({label})"


def check_quant(u: Unit, db_bits, label, ranks):
    """rank-by-rank and all-ranks quantisation against the oracle; returns device codes/scales."""
    want_codes, want_scales = OF.block_quant_all(u.oracle, db_bits)
    nb = want_scales.size
    dbuf = to_dev_bf16(db_bits)
    say(f"quantize all ranks {label}: nb={nb}")
    codes = torch.full((u.total,), 0xAB, dtype=torch.uint8, device="cuda")
    scales = torch.full((max(nb, 1),), float("nan"), dtype=torch.float32, device="cuda")
    B.rs_quantize(u.plan, -1, dbuf, codes, scales)
    torch.cuda.synchronize()
    got_s = scales.cpu().numpy()[:nb]
    assert np.array_equal(got_s.view(np.uint32), want_scales.view(np.uint32)), f"scales differ ({label})"
    got_c = codes.cpu().numpy()
    if not np.array_equal(got_c, want_codes):
        bad = np.flatnonzero(got_c != want_codes)
        raise AssertionError(f"codes differ ({label}) at {bad[:8]}: got {got_c[bad[:8]]} want {want_codes[bad[:8]]}")
    for k in ranks:
        say(f"quantize rank {k} {label}")
        lo, hi = u.oracle.scale_range(k)
        assert B.rs_plan_scale_range(u.plan, k) == (lo, hi)
        c = torch.full((u.S,), 0xCD, dtype=torch.uint8, device="cuda")
        s = torch.full((max(hi - lo, 1),), float("nan"), dtype=torch.float32, device="cuda")
        B.rs_quantize(u.plan, k, dbuf[k * u.S:(k + 1) * u.S], c, s)
        torch.cuda.synchronize()
        oc, os_ = OF.block_quant_shard(u.oracle, k, db_bits[k * u.S:(k + 1) * u.S])
        assert np.array_equal(c.cpu().numpy(), oc), f"rank {k} codes differ ({label})"
        assert np.array_equal(s.cpu().numpy()[:hi - lo].view(np.uint32), os_.view(np.uint32))
    return codes, scales, want_codes, want_scales


def check_dequant_unpack(u: Unit, codes, scales, want_codes, want_scales, label):
    say(f"dequant_unpack {label}")
    outs = [torch.full((s.e,), 0x7FC0, dtype=torch.int16, device="cuda").view(torch.bfloat16) for s in u.specs]
    B.rs_unpack(u.plan, codes, scales, u.table(outs))
    torch.cuda.synchronize()
    want = OF.dequant_unpack(u.oracle, want_codes, want_scales)
    for i, (o, w) in enumerate(zip(outs, want)):
        assert np.array_equal(bits_of(o), w), f"dequant_unpack tensor {i} differs ({label})"
    say(f"unpack_f32 {label}")
    holders = [torch.full((s.e + 3,), float("nan"), dtype=torch.float32, device="cuda") for s in u.specs]
    outs32 = [h[1:1 + s.e] for h, s in zip(holders, u.specs)]          # 4-byte aligned views only
    B.rs_unpack_f32(u.plan, codes, scales, u.table(outs32))
    torch.cuda.synchronize()
    for i, (o, w, h) in enumerate(zip(outs32, OF.dequant_unpack_f32(u.oracle, want_codes, want_scales), holders)):
        assert np.array_equal(o.cpu().numpy().view(np.uint32), w.view(np.uint32)), f"unpack_f32 tensor {i} ({label})"
        edge = h.cpu().numpy()
        assert np.isnan(edge[0]) and np.all(np.isnan(edge[1 + w.size:]))
    aligned = [torch.full((s.e,), float("nan"), dtype=torch.float32, device="cuda") for s in u.specs]
    B.rs_unpack_f32(u.plan, codes, scales, u.table(aligned))
    torch.cuda.synchronize()
    for i, (o, o1) in enumerate(zip(aligned, outs32)):
        assert torch.equal(o.view(torch.int32), o1.contiguous().view(torch.int32)), f"unpack_f32 aligned {i} ({label})"


# ---------------------------------------------------------------------------------------------
# config 1: toy unit, everything, every rank
# ---------------------------------------------------------------------------------------------

def test_config1_all_ops():
    wl = WORKLOADS[1]
    u = Unit.from_workload(wl)
    try:
        params = gen_params(wl, seed=1)
        _, db_bits = check_pack_unpack(u, params, "cfg1")
        for k in range(wl.world):
            parts = np.stack([gen_partial(wl, 1, w, u.S, unit=k) for w in range(wl.world)])
            check_reduce(u, k, parts, "cfg1")
            check_reduce_quant(u, k, parts, "cfg1")
        c, s, wc, ws = check_quant(u, db_bits, "cfg1", range(wl.world))
        check_dequant_unpack(u, c, s, wc, ws, "cfg1")
    finally:
        u.close()


def test_e4m3_encode_every_bf16_value():
    """All finite bf16 values with |x| <= 448 as quantisation inputs at scale exactly 1
    (every block also holds 448, so amax/448 = 1): the hardware convert must agree with the
    format definition on every one, ties and subnormals included."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    x = OD.bf16_bits_to_f32(bits)
    bits = bits[np.isfinite(x) & (np.abs(x) <= 448.0)]
    per = 127
    nblk = -(-bits.size // per)
    data = np.full(nblk * 128, 0x43E0, dtype=np.uint16)         # 448.0
    body = np.zeros(nblk * per, dtype=np.uint16)
    body[:bits.size] = bits
    data.reshape(nblk, 128)[:, :per] = body.reshape(nblk, per)
    for tensors, label in [([(data.size, 0, MODE_1x128)], "1-D runs"),
                           ([(nblk, 128, MODE_1x128)], "row runs"),
                           ([(data.size // 128, 128, MODE_128x128)], "tiles")]:
        u = Unit(tensors, 1)
        try:
            db = OD.ragged_pack([data], u.oracle.offsets, u.total)
            c, s, wc, ws = check_quant(u, db, f"exhaustive {label}", [0])
            if label != "tiles":
                assert np.all(ws == 1.0)
            check_dequant_unpack(u, c, s, wc, ws, f"exhaustive {label}")
        finally:
            u.close()


def test_e4m3_ties_and_neighbours_in_fp32():
    """y = x / scale lands on (and one ulp around) every midpoint between adjacent E4M3 values:
    choose scale = 2^k so y is exact, x = midpoint * 2^k."""
    tab = OF.decode_table()[:0x7F].astype(np.float64)
    mids = (tab[:-1] + tab[1:]) / 2
    vals = []
    for kexp in (-3, 0, 5):
        for m in mids:
            for v in (m, -m):
                vals.append(v * 2.0 ** kexp)
    # bf16 can hold every midpoint (5 significant bits); neighbours come from the exhaustive test
    arr = np.array(vals, dtype=np.float32)
    bits = (arr.view(np.uint32) >> 16).astype(np.uint16)
    assert np.array_equal(OD.bf16_bits_to_f32(bits), arr)
    per = len(mids) * 2
    blocks = []
    for i, kexp in enumerate((-3, 0, 5)):
        chunk = bits[i * per:(i + 1) * per]
        for a in range(0, per, 127):
            blk = np.zeros(128, dtype=np.uint16)
            part = chunk[a:a + 127]
            blk[:part.size] = part
            blk[127] = (np.array([448.0 * 2.0 ** kexp], dtype=np.float32).view(np.uint32) >> 16).astype(np.uint16)[0]
            blocks.append(blk)
    data = np.concatenate(blocks)
    u = Unit([(data.size, 0, MODE_1x128)], 1)
    try:
        db = OD.ragged_pack([data], u.oracle.offsets, u.total)
        check_quant(u, db, "ties", [0])
    finally:
        u.close()


def test_zero_blocks_negative_zero_and_tiny_values():
    rows, cols = 300, 384
    rng_bits = normal_bf16(7, 0, 2, 0, rows * cols, 0.02).reshape(rows, cols)
    rng_bits[128:256, 128:256] = 0                 # an all-zero tile: scale 0, codes 0
    rng_bits[0:128, 0:128] = 0x8000                # all negative zeros: still scale 0, codes 0x00
    rng_bits[0, 256] = 0x0001                      # smallest bf16 subnormal next to normal values
    rng_bits[1, 256] = 0x8001
    rng_bits[256:, 256:] = 0x0003                  # a tile of tiny subnormals only (amax tiny)
    vec = normal_bf16(7, 0, 2, 1, 1000, 1e-30)     # 1-D runs with very small magnitudes
    vec[128:256] = 0
    u = Unit([(rows, cols, MODE_128x128), (1000, 0, MODE_1x128)], 2)
    try:
        db = OD.ragged_pack([rng_bits.reshape(-1), vec], u.oracle.offsets, u.total)
        c, s, wc, ws = check_quant(u, db, "zeros/tiny", range(2))
        check_dequant_unpack(u, c, s, wc, ws, "zeros/tiny")
    finally:
        u.close()


def test_reduce_quantize_special_blocks():
    """Blocks whose mean is all zero, all negative zero, tiny, or so tiny that the scale
    underflows (amax = 2^-142 from one bf16 subnormal among 512 partials), next to ordinary ones;
    one partial (the mean is the partial itself) and a count that is no multiple of 8."""
    rows, cols = 260, 256
    for W in (1, 13, 512):
        u = Unit([(rows, cols, MODE_128x128), (700, 0, MODE_1x128)], W)      # W partials = W ranks
        try:
            S = u.S
            busy = [k for k in range(W) if u.oracle.rank_segments(k)]
            idle = [k for k in range(W) if not u.oracle.rank_segments(k)]
            for k in busy[:4] + idle[:1]:
                parts = np.stack([normal_bf16(31, W, k, w, S, 1e-3) for w in range(W)])
                for t, src_off, dst_off, n in u.oracle.rank_segments(k):
                    if t == 0:
                        region = parts[:, dst_off:dst_off + n].reshape(W, -1, cols)
                        assert np.shares_memory(region, parts)
                        region[:, :, 0:128] = 0                    # zero tiles
                        region[:, :, 128:256] = 0x8000             # negative zeros ...
                        region[0, 0, 128] = 0x0001                 # ... and one subnormal: amax = 2^-133 / W
                        if region.shape[1] > 128:                  # a second row of tiles keeps ordinary values
                            region[:, 128:, :] = normal_bf16(31, W, k, 999, (region.shape[1] - 128) * cols,
                                                             1e-3).reshape(1, -1, cols)
                    else:
                        parts[:, dst_off:dst_off + 256] = 0        # a zero run, and a run whose only value
                        parts[W - 1, dst_off + 130] = 0x8001       # is a negative subnormal
                check_reduce_quant(u, k, parts, f"special W={W}")
        finally:
            u.close()


RAGGED_UNITS = [
    # (tensors, world, align_bytes, min_itemsize, tensor_align): odd pitches, partial tiles,
    # rows that are not 16-byte multiples, paper-literal A = 1 (nothing vector-aligned)
    ([(257, 130, MODE_128x128), (5, 0, MODE_1x128), (129, 7, MODE_128x128), (300, 0, MODE_1x128)], 3, 16, 1, 0),
    ([(64, 200, MODE_1x128), (33, 136, MODE_1x128), (1, 0, MODE_1x128), (130, 129, MODE_128x128)], 5, 16, 1, 0),
    ([(257, 130, MODE_128x128), (383, 0, MODE_1x128), (129, 8, MODE_128x128)], 4, 16, 1, 1),
    ([(17, 24, MODE_1x128), (250, 0, MODE_1x128), (128, 256, MODE_128x128)], 7, 32, 1, 2),
    ([(2048, 0, MODE_1x128)], 16, 16, 1, 0),
    ([(128, 128, MODE_128x128)], 8, 16, 1, 0),                      # most ranks empty
]


@pytest.mark.parametrize("case", range(len(RAGGED_UNITS)))
def test_ragged_units_all_ops(case):
    tensors, world, align, item, A = RAGGED_UNITS[case]
    u = Unit(tensors, world, align, item, A)
    try:
        params = [normal_bf16(11, case, 0, i, s.e, 0.02) for i, s in enumerate(u.specs)]
        _, db_bits = check_pack_unpack(u, params, f"ragged{case}")
        for k in range(world):
            parts = np.stack([normal_bf16(11, case, 1, k * 64 + w, u.S, 1e-3) for w in range(world)])
            check_reduce(u, k, parts, f"ragged{case}")
            check_reduce_quant(u, k, parts, f"ragged{case}")
        c, s, wc, ws = check_quant(u, db_bits, f"ragged{case}", range(world))
        check_dequant_unpack(u, c, s, wc, ws, f"ragged{case}")
    finally:
        u.close()


def test_unaligned_tensor_storage():
    """Sources / destinations that are only element-aligned (views at odd offsets)."""
    tensors = [(130, 136, MODE_128x128), (700, 0, MODE_1x128), (64, 256, MODE_1x128)]
    u = Unit(tensors, 3)
    try:
        params = [normal_bf16(12, 0, 0, i, s.e, 0.02) for i, s in enumerate(u.specs)]
        holders = [torch.zeros(p.size + 8, dtype=torch.bfloat16, device="cuda") for p in params]
        views = []
        for i, (h, p) in enumerate(zip(holders, params)):
            v = h[1 + i:1 + i + p.size]
            v.copy_(to_dev_bf16(p))
            views.append(v)
        dbuf = torch.full((u.total,), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
        say("pack from unaligned sources")
        B.rs_pack(u.plan, u.table(views), dbuf)
        torch.cuda.synchronize()
        want = OD.ragged_pack(params, u.oracle.offsets, u.total)
        assert np.array_equal(bits_of(dbuf), want)
        outs_h = [torch.zeros(p.size + 8, dtype=torch.bfloat16, device="cuda") for p in params]
        outs = [h[3:3 + p.size] for h, p in zip(outs_h, params)]
        say("unpack_bf16 to unaligned destinations")
        B.rs_unpack_bf16(u.plan, dbuf, u.table(outs))
        torch.cuda.synchronize()
        for o, p, h in zip(outs, params, outs_h):
            assert np.array_equal(bits_of(o), p)
            assert bits_of(h)[:3].tolist() == [0, 0, 0] and bits_of(h)[3 + p.size:].tolist() == [0] * 5
        wc, ws = OF.block_quant_all(u.oracle, want)
        codes = torch.from_numpy(wc).cuda()
        scales = torch.from_numpy(ws).cuda()
        outs_h = [torch.zeros(p.size + 8, dtype=torch.bfloat16, device="cuda") for p in params]
        outs = [h[5:5 + p.size] for h, p in zip(outs_h, params)]
        say("dequant_unpack to unaligned destinations")
        B.rs_unpack(u.plan, codes, scales, u.table(outs))
        torch.cuda.synchronize()
        for o, w, h in zip(outs, OF.dequant_unpack(u.oracle, wc, ws), outs_h):
            assert np.array_equal(bits_of(o), w)
            assert bits_of(h)[:5].tolist() == [0] * 5 and bits_of(h)[5 + w.size:].tolist() == [0] * 3
    finally:
        u.close()


@pytest.mark.parametrize("W", [1, 2, 3, 8, 9, 15, 16, 17, 100, 128, 131, 257])
def test_reduce_world_sizes_and_special_cases(W):
    tensors = [(3000, 0, MODE_1x128), (70, 130, MODE_1x128)]
    u = Unit(tensors, W)
    try:
        rank = W // 2
        parts = np.stack([normal_bf16(13, W, 1, w, u.S, 1e-3) for w in range(W)])
        got = check_reduce(u, rank, parts, f"W={W}")
        if W == 1:      # exact widening of the only partial
            pay = got != 0
            assert np.array_equal(got[pay], OD.bf16_bits_to_f32(parts[0])[pay])
        if W in (2, 8, 16):   # equal partials, W a power of two: the value itself
            same = np.repeat(parts[:1], W, axis=0)
            got = check_reduce(u, rank, same, f"W={W} equal", poison_padding=False)
            segs = u.oracle.rank_segments(rank)
            for _, _, d, n in segs:
                assert np.array_equal(got[d:d + n], OD.bf16_bits_to_f32(parts[0, d:d + n]))
    finally:
        u.close()


@pytest.mark.parametrize("rows", [1, 3, 12, 200])
def test_reduce_over_a_row_count_other_than_the_world_size(rows):
    """The 2-D gradient reduction of an N-D buffer: a region of a 4-rank plan receives one
    partial per (rank, replica) pair, or one per replica."""
    wl = WORKLOADS[1]
    u = Unit.from_workload(wl)
    try:
        for k in (0, wl.world - 1):
            parts = np.stack([normal_bf16(33, rows, k, w, u.S, 1e-3) for w in range(rows)])
            check_reduce(u, k, parts, f"rows={rows}")
        with pytest.raises(B.RaggedShardError) as e:
            B.rs_reduce_rows(u.plan, 0, torch.zeros(8, device="cuda"), 0, u.S, torch.zeros(8, device="cuda"))
        assert e.value.code == B.RS_EINVAL
    finally:
        u.close()


def test_reduce_row_stride_and_large_magnitudes():
    W = 12
    u = Unit([(5000, 0, MODE_1x128)], 3)
    try:
        S = u.S
        stride = S + 64
        big = np.stack([normal_bf16(14, 0, 1, w, S, 3.0e4) for w in range(W)])   # cancellation-prone
        buf = torch.zeros(W * stride, dtype=torch.bfloat16, device="cuda")
        buf.view(W, stride)[:, :S].copy_(to_dev_bf16(big.reshape(-1)).view(W, S))
        out = torch.empty(S, dtype=torch.float32, device="cuda")
        say("reduce with a row stride > S")
        B.rs_reduce(u.plan, 1, buf, stride, out)
        torch.cuda.synchronize()
        # W here is the plan's world (3): only the first 3 rows are read
        want = OD.shard_reduce(big[:3], u.oracle.rank_segments(1))
        bound = REDUCE_TOL * OD.shard_reduce_abs_sum(big[:3])
        assert np.all(np.abs(out.cpu().numpy().astype(np.float64) - want) <= bound)
        ordered = OD.shard_reduce_f32_ordered(big[:3], u.oracle.rank_segments(1))
        assert np.array_equal(out.cpu().numpy().view(np.uint32), ordered.view(np.uint32))
    finally:
        u.close()


def test_device_argument_errors():
    u = Unit([(256, 128, MODE_128x128)], 2)
    w = Unit([(64, 64, MODE_WHOLE)], 2, 16, 2)
    try:
        x = torch.zeros(u.total + 8, dtype=torch.bfloat16, device="cuda")
        tab = u.table([torch.zeros(256 * 128, dtype=torch.bfloat16, device="cuda")])
        with pytest.raises(B.RaggedShardError) as e:
            B.rs_pack(u.plan, tab, x[1:])                       # misaligned DBuffer
        assert e.value.code == B.RS_EALIGN
        with pytest.raises(B.RaggedShardError) as e:
            B.rs_reduce(u.plan, 2, x, u.S, torch.zeros(u.S, device="cuda"))   # rank out of range
        assert e.value.code == B.RS_EINVAL
        with pytest.raises(B.RaggedShardError) as e:
            B.rs_reduce(u.plan, 0, x, u.S + 3, torch.zeros(u.S, device="cuda"))
        assert e.value.code == B.RS_EALIGN
        with pytest.raises(B.RaggedShardError) as e:
            B.rs_reduce(u.plan, 0, x, u.S - 8, torch.zeros(u.S, device="cuda"))
        assert e.value.code == B.RS_EINVAL
        codes = torch.zeros(w.total, dtype=torch.uint8, device="cuda")
        with pytest.raises(B.RaggedShardError) as e:
            B.rs_quantize(w.plan, 0, x, codes, torch.zeros(4, device="cuda"))  # whole-matrix plan
        assert e.value.code == B.RS_EUNSUPPORTED
        with pytest.raises(B.RaggedShardError) as e:
            B.rs_pack(w.plan, tab, x)                           # table made for another plan
        assert e.value.code == B.RS_EINVAL
        # the fused reduce + quantise checks what both of its halves check
        sc, mean = torch.zeros(8, device="cuda"), torch.zeros(u.S + 4, device="cuda")
        ucodes = torch.zeros(u.S, dtype=torch.uint8, device="cuda")
        for args, code in [((u.plan, 2, x, u.S, ucodes, sc), B.RS_EINVAL),             # rank out of range
                           ((u.plan, 0, x, u.S - 8, ucodes, sc), B.RS_EINVAL),         # rows overlap
                           ((u.plan, 0, x, u.S + 3, ucodes, sc), B.RS_EALIGN),         # row stride
                           ((u.plan, 0, x[1:], u.S, ucodes, sc), B.RS_EALIGN),         # partials
                           ((u.plan, 0, x, u.S, ucodes, sc, mean[1:]), B.RS_EALIGN),   # mean buffer
                           ((w.plan, 0, x, w.S, codes, sc), B.RS_EUNSUPPORTED)]:       # no FP8 blocks
            with pytest.raises(B.RaggedShardError) as e:
                B.rs_reduce_quantize(*args)
            assert e.value.code == code, args[1:4]
        with pytest.raises(B.RaggedShardError) as e:
            B.rs_reduce_rows(u.plan, 0, x, 1 << 25, u.S, torch.zeros(u.S, device="cuda"))
        assert e.value.code == B.RS_EINVAL
    finally:
        u.close()
        w.close()


def test_reduce_long_region_two_granule_workgroups():
    """Regions of 4096 granules or more are reduced by 512-lane workgroups that take two granules
    each and keep the next eight rows in flight; check that path element by element, ragged tail
    and padding included."""
    W = 3
    u = Unit([(9_000_001, 0, MODE_1x128), (700, 136, MODE_128x128), (16_500_000, 0, MODE_1x128)], W)
    try:
        assert -(-u.S // 2048) >= 4096
        for rank in range(W):
            parts = np.stack([normal_bf16(15, rank, 1, w, u.S, 1e-3) for w in range(W)])
            check_reduce(u, rank, parts, f"long region rank {rank}")
    finally:
        u.close()


def test_reduce_long_region_many_partials():
    """The long-region kernel with more rows than one batch of eight, W not a multiple of 8."""
    W = 35
    u = Unit([(W * 8_400_000 + 77, 0, MODE_1x128)], W)
    try:
        assert -(-u.S // 2048) >= 4096
        rank = W - 1
        parts = np.stack([normal_bf16(16, rank, 1, w, u.S, 1e-3) for w in range(W)])
        check_reduce(u, rank, parts, f"long region, W={W}, rank {rank}")
    finally:
        u.close()


def test_quantize_batch_equals_per_unit_quantize():
    """rs_quantize_batch over several units that share a plan: every unit's codes and scales
    equal the oracle's shard quantisation bit for bit (and hence rs_quantize's)."""
    tensors = [(300, 384, MODE_128x128), (1000, 0, MODE_1x128), (257, 130, MODE_128x128), (64, 256, MODE_1x128)]
    u = Unit(tensors, 3)
    try:
        n_units = 5
        for rank in range(3):
            lo, hi = u.oracle.scale_range(rank)
            dbs, shards, codes, scales = [], [], [], []
            for unit in range(n_units):
                params = [normal_bf16(16, unit, 0, i, s.e, 0.02 * (unit + 1)) for i, s in enumerate(u.specs)]
                db = OD.ragged_pack(params, u.oracle.offsets, u.total)
                dbs.append(db)
                shards.append(to_dev_bf16(db[rank * u.S:(rank + 1) * u.S].copy()))
                codes.append(torch.full((u.S,), 0xEE, dtype=torch.uint8, device="cuda"))
                scales.append(torch.full((max(1, hi - lo),), float("nan"), dtype=torch.float32, device="cuda"))
            say(f"quantize_batch rank {rank}: {n_units} units")
            batch = B.rs_shard_batch_create(u.plan, rank, shards, codes, scales)
            B.rs_quantize_batch(u.plan, batch)
            torch.cuda.synchronize()
            B.rs_shard_batch_destroy(batch)
            for unit in range(n_units):
                oc, os_ = OF.block_quant_shard(u.oracle, rank, dbs[unit][rank * u.S:(rank + 1) * u.S])
                assert np.array_equal(codes[unit].cpu().numpy(), oc), f"unit {unit} codes"
                assert np.array_equal(scales[unit].cpu().numpy()[:hi - lo].view(np.uint32), os_.view(np.uint32))
        with pytest.raises(B.RaggedShardError) as e:
            B.rs_shard_batch_create(u.plan, 3, shards, codes, scales)
        assert e.value.code == B.RS_EINVAL
    finally:
        u.close()


@pytest.mark.parametrize("long_region", [False, True])
def test_reduce_batch_equals_per_unit_reduce(long_region):
    """rs_reduce_batch over several units that share a plan: every unit's mean is within the
    tolerance of the float64 definition, equals the stated fp32 order bit for bit and equals
    rs_reduce on the same partials; short regions (256-lane workgroups) and long ones (512)."""
    if long_region:
        W, n_units = 3, 3
        tensors = [(9_000_001, 0, MODE_1x128), (700, 136, MODE_128x128), (16_500_000, 0, MODE_1x128)]
    else:
        W, n_units = 6, 5
        tensors = [(300, 384, MODE_128x128), (1000, 0, MODE_1x128), (257, 130, MODE_128x128), (64, 256, MODE_1x128)]
    u = Unit(tensors, W)
    try:
        assert (-(-u.S // 2048) >= 4096) == long_region
        stride = u.S + 24          # rows further apart than S, as a strided view would be
        for rank in (0, W - 1):
            segs = u.oracle.rank_segments(rank)
            hosts, devs, outs, singles = [], [], [], []
            for unit in range(n_units):
                parts = np.stack([normal_bf16(21, unit, 1, 100 * rank + w, u.S, 1e-3 * (unit + 1)) for w in range(W)])
                padded = np.zeros((W, stride), dtype=np.uint16)
                padded[:, :u.S] = parts
                padded[:, u.S:] = 0x7fc0          # NaN between the rows: must never be read into a sum
                hosts.append(parts)
                devs.append(to_dev_bf16(padded.reshape(-1)))
                outs.append(torch.full((u.S,), float("nan"), dtype=torch.float32, device="cuda"))
                singles.append(torch.full((u.S,), float("nan"), dtype=torch.float32, device="cuda"))
            say(f"reduce_batch rank {rank}: {n_units} units, long={long_region}")
            batch = B.rs_partials_batch_create(u.plan, rank, devs, stride, outs)
            B.rs_reduce_batch(u.plan, batch)
            for unit in range(n_units):
                B.rs_reduce(u.plan, rank, devs[unit], stride, singles[unit])
            torch.cuda.synchronize()
            B.rs_partials_batch_destroy(batch)
            for unit in range(n_units):
                got = outs[unit].cpu().numpy()
                assert np.array_equal(got.view(np.uint32), singles[unit].cpu().numpy().view(np.uint32)), f"unit {unit}"
                want = OD.shard_reduce(hosts[unit], segs)
                assert np.all(np.abs(got.astype(np.float64) - want) <= REDUCE_TOL * OD.shard_reduce_abs_sum(hosts[unit]))
                ordered = OD.shard_reduce_f32_ordered(hosts[unit], segs)
                assert np.array_equal(got.view(np.uint32), ordered.view(np.uint32)), f"unit {unit} order"
        x = torch.zeros(W * stride, dtype=torch.bfloat16, device="cuda")
        o = torch.zeros(u.S, dtype=torch.float32, device="cuda")
        for args, code in [((u.plan, W, [x], stride, [o]), B.RS_EINVAL),            # rank out of range
                           ((u.plan, 0, [x], u.S - 8, [o]), B.RS_EINVAL),           # rows overlap
                           ((u.plan, 0, [x], stride + 4, [o]), B.RS_EALIGN),        # stride not 16-byte
                           ((u.plan, 0, [x[1:]], stride, [o]), B.RS_EALIGN)]:       # partials misaligned
            with pytest.raises(B.RaggedShardError) as e:
                B.rs_partials_batch_create(*args)
            assert e.value.code == code
    finally:
        u.close()


@pytest.mark.parametrize("order", [1, 2, 3])
def test_reordered_plans_all_ops(order):
    """Plans whose buffer order differs from the caller's tensor order (sorted by block size, by
    shape, best of three): pointer tables, offsets and the scale layout must all follow."""
    wl = WORKLOADS[1]
    tensors = [(t.rows, t.cols, t.mode) for t in wl.tensors] + [(200, 0, MODE_1x128), (64, 520, MODE_1x128)]
    u = Unit(tensors, 5, order=order)
    try:
        if order != 3:
            assert u.oracle.buffer_order() != list(range(len(tensors)))
        params = [normal_bf16(17, order, 0, i, s.e, 0.02) for i, s in enumerate(u.specs)]
        _, db_bits = check_pack_unpack(u, params, f"order{order}")
        for k in range(5):
            parts = np.stack([normal_bf16(17, order, 1, k * 8 + w, u.S, 1e-3) for w in range(5)])
            check_reduce(u, k, parts, f"order{order}")
            check_reduce_quant(u, k, parts, f"order{order}")
        c, s, wc, ws = check_quant(u, db_bits, f"order{order}", range(5))
        check_dequant_unpack(u, c, s, wc, ws, f"order{order}")
    finally:
        u.close()


def test_rooted_plan_all_ops():
    """RaggedShard(r_t): every tensor whole on its root device, some devices empty, tensors of one
    device back to back.  All four kernels run from the same tables as for a balanced plan."""
    tensors = [(300, 136, MODE_128x128), (200, 0, MODE_1x128), (64, 520, MODE_1x128), (129, 256, MODE_128x128),
               (1000, 0, MODE_1x128), (40, 128, MODE_128x128), (77, 24, MODE_1x128)]
    roots = [3, 0, 3, 1, 1, 5, 0]
    u = Unit(tensors, 6, roots=roots)
    try:
        assert B.rs_plan_order(u.plan) == [1, 6, 3, 4, 0, 2, 5]
        params = [normal_bf16(23, 0, 0, i, s.e, 0.02) for i, s in enumerate(u.specs)]
        _, db_bits = check_pack_unpack(u, params, "rooted")
        for k in range(6):
            parts = np.stack([normal_bf16(23, 0, 1, k * 8 + w, u.S, 1e-3) for w in range(6)])
            check_reduce(u, k, parts, "rooted")
            check_reduce_quant(u, k, parts, "rooted")
        c, s, wc, ws = check_quant(u, db_bits, "rooted", range(6))
        check_dequant_unpack(u, c, s, wc, ws, "rooted")
    finally:
        u.close()


def test_redistribute_to_roots_and_back():
    """Algorithm 2's data path on one device: the momentum of a unit sits in the balanced buffer
    P; redistributing to RaggedShard(r) is the group copy-out of P into views of the rooted
    buffer Q (one launch, no intermediate tensors), and the way back is P's copy-in from the same
    views.  Roots come from the library's SelectRoot."""
    wl = WORKLOADS[1]
    tensors = [(t.rows, t.cols, MODE_WHOLE if t.cols else t.mode) for t in wl.tensors]
    mats = [i for i, t in enumerate(tensors) if t[1] > 0]
    roots, _ = B.rs_select_roots(tensors, 3)
    roots = [r if r >= 0 else 0 for r in roots]            # the vectors stay with device 0
    p = Unit([(t.rows, t.cols, t.mode) for t in wl.tensors], wl.world, 16, 2)
    q = Unit(tensors, 3, 16, 2, roots=roots)
    try:
        assert len({roots[i] for i in mats}) == min(3, len(mats))
        params = [normal_bf16(29, 1, 0, i, s.e, 0.02) for i, s in enumerate(p.specs)]
        p_bits = OD.ragged_pack(params, p.oracle.offsets, p.total)
        q_bits = OD.ragged_pack(params, q.oracle.offsets, q.total)
        pbuf = to_dev_bf16(p_bits)
        qbuf = torch.full((q.total,), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
        views = [qbuf[l:l + s.e] for l, s in zip(q.oracle.offsets, q.specs)]
        say("redistribute P -> Q")
        B.rs_group_zero(q.plan, qbuf)
        B.rs_unpack_bf16(p.plan, pbuf, p.table(views))
        torch.cuda.synchronize()
        assert np.array_equal(bits_of(qbuf), q_bits)
        say("redistribute Q -> P")
        back = torch.full((p.total,), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
        B.rs_pack(p.plan, p.table(views), back)
        torch.cuda.synchronize()
        assert np.array_equal(bits_of(back), p_bits)
    finally:
        p.close()
        q.close()


def test_whole_path_replays_from_a_hip_graph():
    """Device calls neither allocate nor synchronise, so the whole path (pack, reduce, quantise,
    unpack, Adam step) can be captured once and replayed: three replays on fresh inputs, with eager
    work and synchronisations in between, each compared with the eager result of the same inputs."""
    tensors = [(512, 256, MODE_128x128), (300, 0, MODE_1x128), (257, 136, MODE_128x128), (128, 384, MODE_128x128)]
    W, rank = 4, 1
    u = Unit(tensors, W)
    try:
        S, total = u.S, u.total
        nb = B.rs_plan_num_scales(u.plan)
        lo, hi = B.rs_plan_state_range(u.plan, rank)

        def buffers():
            return dict(
                src=[torch.zeros(s.e, dtype=torch.bfloat16, device="cuda") for s in u.specs],
                dst=[torch.zeros(s.e, dtype=torch.bfloat16, device="cuda") for s in u.specs],
                dbuf=torch.zeros(total, dtype=torch.bfloat16, device="cuda"),
                parts=torch.zeros(W * S, dtype=torch.bfloat16, device="cuda"),
                grad=torch.zeros(S, dtype=torch.float32, device="cuda"),
                codes=torch.zeros(total, dtype=torch.uint8, device="cuda"),
                scales=torch.zeros(nb, dtype=torch.float32, device="cuda"),
                master=torch.zeros(S, dtype=torch.float32, device="cuda"),
                param=torch.zeros(S, dtype=torch.bfloat16, device="cuda"),
                mc=torch.zeros(S, dtype=torch.int8, device="cuda"), vc=torch.zeros(S, dtype=torch.uint8, device="cuda"),
                am=torch.zeros(max(hi - lo, 1), dtype=torch.float32, device="cuda"),
                av=torch.zeros(max(hi - lo, 1), dtype=torch.float32, device="cuda"))

        def path(b, tab_src, tab_dst, stream=None):
            B.rs_pack(u.plan, tab_src, b["dbuf"], stream)
            B.rs_reduce(u.plan, rank, b["parts"], S, b["grad"], stream)
            B.rs_adam8_step(u.plan, rank, (1e-3, 0.9, 0.95, 1e-8, 0.01, 3), b["grad"], b["master"], b["param"],
                            b["mc"], b["vc"], b["am"], b["av"], stream)
            B.rs_quantize(u.plan, -1, b["dbuf"], b["codes"], b["scales"], stream)
            B.rs_unpack(u.plan, b["codes"], b["scales"], tab_dst, stream)

        g_buf, e_buf = buffers(), buffers()
        g_src, g_dst = u.table(g_buf["src"]), u.table(g_buf["dst"])
        e_src, e_dst = u.table(e_buf["src"]), u.table(e_buf["dst"])
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            path(g_buf, g_src, g_dst, side)          # warm-up outside capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        say("capturing the path into a HIP graph")
        with torch.cuda.graph(graph):
            path(g_buf, g_src, g_dst)
        for rep in range(3):
            params = [normal_bf16(40, rep, 0, i, s.e, 0.02) for i, s in enumerate(u.specs)]
            parts = np.stack([normal_bf16(40, rep, 1, w, S, 1e-3) for w in range(W)])
            for b in (g_buf, e_buf):
                for t, p in zip(b["src"], params):
                    t.copy_(to_dev_bf16(p))
                b["parts"].copy_(to_dev_bf16(parts.reshape(-1)))
                for k in ("master", "mc", "vc", "am", "av"):
                    b[k].zero_()
                b["master"].add_(0.01 * (rep + 1))
            torch.cuda.synchronize()
            say(f"replay {rep}")
            graph.replay()
            path(e_buf, e_src, e_dst)
            torch.cuda.synchronize()
            for k in ("dbuf", "grad", "codes", "scales", "master", "param", "mc", "vc", "am", "av"):
                a, c = g_buf[k], e_buf[k]
                if a.dtype == torch.bfloat16:
                    a, c = a.view(torch.int16), c.view(torch.int16)
                elif a.dtype == torch.float32:
                    a, c = a.view(torch.int32), c.view(torch.int32)
                assert torch.equal(a, c), f"{k} differs on replay {rep}"
            for a, c in zip(g_buf["dst"], e_buf["dst"]):
                assert torch.equal(a.view(torch.int16), c.view(torch.int16)), f"unpacked tensor differs on replay {rep}"
            # and the eager result is the oracle's (pack only: the other ops are checked elsewhere)
            assert np.array_equal(bits_of(e_buf["dbuf"]), OD.ragged_pack(params, u.oracle.offsets, total))
    finally:
        u.close()


def test_one_plan_serves_two_threads_on_two_streams():
    """An uploaded plan and its tables are read-only: two host threads, each with a stream and
    buffers of its own, run the path at the same time and must each get the single-stream result."""
    import threading

    tensors = [(512, 256, MODE_128x128), (300, 0, MODE_1x128), (257, 136, MODE_128x128), (384, 384, MODE_128x128)]
    W, reps = 4, 10
    u = Unit(tensors, W)
    try:
        S, total = u.S, u.total
        nb = B.rs_plan_num_scales(u.plan)

        def make(seed):
            params = [normal_bf16(70, seed, 0, i, s.e, 0.02) for i, s in enumerate(u.specs)]
            parts = np.stack([normal_bf16(70, seed, 1, w, S, 1e-3) for w in range(W)])
            b = dict(src=[to_dev_bf16(p) for p in params], parts=to_dev_bf16(parts.reshape(-1)),
                     dst=[torch.zeros(s.e, dtype=torch.bfloat16, device="cuda") for s in u.specs],
                     dbuf=torch.zeros(total, dtype=torch.bfloat16, device="cuda"),
                     grad=torch.zeros(S, dtype=torch.float32, device="cuda"),
                     codes=torch.zeros(total, dtype=torch.uint8, device="cuda"),
                     scales=torch.zeros(nb, dtype=torch.float32, device="cuda"))
            b["tab_src"], b["tab_dst"] = u.table(b["src"]), u.table(b["dst"])
            return b

        def path(b, rank, stream):
            B.rs_pack(u.plan, b["tab_src"], b["dbuf"], stream)
            B.rs_reduce(u.plan, rank, b["parts"], S, b["grad"], stream)
            B.rs_quantize(u.plan, -1, b["dbuf"], b["codes"], b["scales"], stream)
            B.rs_unpack(u.plan, b["codes"], b["scales"], b["tab_dst"], stream)

        def snapshot(b):
            return [b[k].clone() for k in ("dbuf", "grad", "codes", "scales")] + [t.clone() for t in b["dst"]]

        work = [make(0), make(1)]
        want = []
        for i, b in enumerate(work):
            path(b, i, None)
            torch.cuda.synchronize()
            want.append(snapshot(b))
            for k in ("dbuf", "grad", "codes", "scales"):
                b[k].view(torch.uint8).fill_(0x33)
            for t in b["dst"]:
                t.view(torch.uint8).fill_(0x33)
        torch.cuda.synchronize()
        streams = [torch.cuda.Stream(), torch.cuda.Stream()]
        errors = []

        def worker(i):
            try:
                torch.cuda.set_device(0)
                for _ in range(reps):
                    path(work[i], i, streams[i])
            except Exception as exc:      # surfaced in the main thread
                errors.append(exc)

        say("two threads, two streams")
        threads = [threading.Thread(target=worker, args=(i,)) for i in range(2)]
        for t in threads:
            t.start()
        for t in threads:
            t.join(timeout=100)
            assert not t.is_alive()
        torch.cuda.synchronize()
        assert not errors, errors
        for i, b in enumerate(work):
            for got, exp in zip(snapshot(b), want[i]):
                assert torch.equal(got.view(torch.uint8), exp.view(torch.uint8)), f"thread {i} result differs"
    finally:
        u.close()


def random_quantised_unit(rnd):
    """A random unit of tensors that carry FP8 blocks: odd pitches, short tensors, partial tiles."""
    n = rnd.randint(1, 7)
    tensors = []
    for _ in range(n):
        kind = rnd.random()
        if kind < 0.3:
            tensors.append((rnd.randint(1, 3000), 0, MODE_1x128))
        elif kind < 0.7:
            tensors.append((rnd.randint(1, 400), rnd.choice([8, 24, 30, 128, 130, 136, 256, 100, 1100]), MODE_128x128))
        else:
            tensors.append((rnd.randint(1, 60), rnd.choice([8, 40, 128, 200, 333]), MODE_1x128))
    world = rnd.choice([1, 2, 3, 4, 7, 8, 16, 33])
    align, item = rnd.choice([(16, 1), (16, 2), (32, 1)])
    A = rnd.choice([0, 0, 0, 1, 2, 8])
    if A and (align // item) % A:
        A = 0
    return tensors, world, align, item, A


@pytest.mark.parametrize("seed", range(24))
def test_random_units_all_ops(seed):
    import random
    rnd = random.Random(9000 + seed)
    tensors, world, align, item, A = random_quantised_unit(rnd)
    u = Unit(tensors, world, align, item, A, order=rnd.choice([0, 0, 1, 2, 3]))
    try:
        say(f"random unit {seed}: {tensors} W={world} align={align}/{item} A={A} S={u.S}")
        params = [normal_bf16(50, seed, 0, i, s.e, 0.02) for i, s in enumerate(u.specs)]
        _, db_bits = check_pack_unpack(u, params, f"random{seed}")
        ranks = sorted(set(rnd.sample(range(world), min(world, 3)) + [0, world - 1]))
        for k in ranks:
            parts = np.stack([normal_bf16(50, seed, 1, k * 64 + w, u.S, 1e-3) for w in range(world)])
            check_reduce(u, k, parts, f"random{seed}")
            check_reduce_quant(u, k, parts, f"random{seed}")
        c, s, wc, ws = check_quant(u, db_bits, f"random{seed}", ranks)
        check_dequant_unpack(u, c, s, wc, ws, f"random{seed}")
    finally:
        u.close()


@pytest.mark.parametrize("write_means", [False, True])
def test_reduce_quantize_batch_equals_per_unit(write_means):
    """rs_reduce_quantize_batch over several units that share a plan: codes, scales and (when
    asked for) means of every unit equal the oracle's and rs_reduce_quantize's, bit for bit;
    without write_means the mean buffers are left untouched.  Ragged tensors and padding included."""
    W, n_units = 5, 4
    tensors = [(300, 384, MODE_128x128), (1000, 0, MODE_1x128), (257, 130, MODE_128x128), (64, 256, MODE_1x128),
               (77, 24, MODE_1x128)]
    u = Unit(tensors, W)
    try:
        stride = u.S + 16
        for rank in (0, 2, W - 1):
            lo, hi = u.oracle.scale_range(rank)
            hosts, devs, means, codes, scales, shards = [], [], [], [], [], []
            for unit in range(n_units):
                parts = np.stack([normal_bf16(23, unit, 1, 100 * rank + w, u.S, 1e-3 * (unit + 1)) for w in range(W)])
                padded = np.full((W, stride), 0x7fc0, dtype=np.uint16)     # NaN between the rows
                padded[:, :u.S] = parts
                hosts.append(parts)
                devs.append(to_dev_bf16(padded.reshape(-1)))
                means.append(torch.full((u.S,), float("nan"), dtype=torch.float32, device="cuda"))
                codes.append(torch.full((u.S,), 0xEE, dtype=torch.uint8, device="cuda"))
                scales.append(torch.full((max(hi - lo, 1),), float("nan"), dtype=torch.float32, device="cuda"))
                shards.append(torch.zeros(u.S, dtype=torch.bfloat16, device="cuda"))   # required by the batch, not read
            say(f"reduce_quantize_batch rank {rank}: {n_units} units, write_means={write_means}")
            pin = B.rs_partials_batch_create(u.plan, rank, devs, stride, means)
            pout = B.rs_shard_batch_create(u.plan, rank, shards, codes, scales)
            B.rs_reduce_quantize_batch(u.plan, pin, pout, write_means)
            torch.cuda.synchronize()
            for unit in range(n_units):
                want_c, want_s, want_mean = OF.reduce_quant_shard(u.oracle, rank, hosts[unit])
                one_c = torch.full((u.S,), 0xEE, dtype=torch.uint8, device="cuda")
                one_s = torch.full((max(hi - lo, 1),), float("nan"), dtype=torch.float32, device="cuda")
                B.rs_reduce_quantize(u.plan, rank, devs[unit], stride, one_c, one_s)
                torch.cuda.synchronize()
                got_c, got_s = codes[unit].cpu().numpy(), scales[unit].cpu().numpy()[:hi - lo]
                assert np.array_equal(got_c, want_c), f"unit {unit} codes"
                assert np.array_equal(got_s.view(np.uint32), want_s.view(np.uint32)), f"unit {unit} scales"
                assert np.array_equal(got_c, one_c.cpu().numpy())
                assert np.array_equal(got_s.view(np.uint32), one_s.cpu().numpy()[:hi - lo].view(np.uint32))
                got_m = means[unit].cpu().numpy()
                if write_means:
                    assert np.array_equal(got_m.view(np.uint32), want_mean.view(np.uint32)), f"unit {unit} mean"
                else:
                    assert np.all(np.isnan(got_m)), "mean buffers must not be written"
            # batches made for another rank or count are refused
            other = B.rs_shard_batch_create(u.plan, (rank + 1) % W, shards, codes, scales)
            fewer = B.rs_shard_batch_create(u.plan, rank, shards[:2], codes[:2], scales[:2])
            for bad in (other, fewer):
                with pytest.raises(B.RaggedShardError) as e:
                    B.rs_reduce_quantize_batch(u.plan, pin, bad)
                assert e.value.code == B.RS_EINVAL
                B.rs_shard_batch_destroy(bad)
            B.rs_partials_batch_destroy(pin)
            B.rs_shard_batch_destroy(pout)
    finally:
        u.close()
