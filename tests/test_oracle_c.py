"""Two independent oracles held against each other: the numpy oracle and the plain C / OpenMP one
(oracle/c/oracle.c) must agree bit for bit on every operation of the hot path.  The C encoder
works from frexp / nearbyint, the numpy one from a midpoint search: a mistake in either shows."""
import numpy as np
import pytest

from oracle import c_oracle as OC
from oracle import dbuffer as D
from oracle import fp8 as F
from oracle import plan as P
from workloads import WORKLOADS, gen_params, gen_partial, normal_bf16


def toy():
    wl = WORKLOADS[1]
    specs = [P.TensorSpec(t.rows, t.cols, t.mode) for t in wl.tensors]
    return wl, P.make_plan(specs, wl.world, wl.align_bytes, wl.min_itemsize)


def test_scalar_codec_pieces_agree():
    L = OC.lib()
    tab = F.decode_table()
    for c in range(256):
        if (c & 0x7F) == 0x7F:
            continue                                      # the two NaN codes
        assert np.float32(L.oc_e4m3_value(c)) == tab[c], c
    bits = np.arange(0, 1 << 16, dtype=np.uint32).astype(np.uint16)
    x = D.bf16_bits_to_f32(bits)
    x = x[np.isfinite(x) & (np.abs(x) <= 448)]
    rng = np.random.default_rng(1)
    rnd = (rng.standard_normal(20000) * 60).astype(np.float32).clip(-448, 448)
    pos = np.array([F.e4m3_value(c) for c in range(0x7F)], dtype=np.float64)
    mid = ((pos[:-1] + pos[1:]) / 2).astype(np.float32)
    ties = np.concatenate([mid, np.nextafter(mid, np.float32(0)), np.nextafter(mid, np.float32(1e9)), -mid])
    for arr in (x, rnd, ties):
        want = F.encode_e4m3(arr)
        got = np.array([L.oc_e4m3_encode(float(v)) for v in arr], dtype=np.uint8)
        assert np.array_equal(got, want)
    f = np.concatenate([(rng.standard_normal(5000) * 1e-2).astype(np.float32),
                        np.array([1.00390625, 1.01171875, 0.0, -0.0, 3e-39], dtype=np.float32)])
    assert np.array_equal(np.array([L.oc_f32_to_bf16(float(v)) for v in f], dtype=np.uint16), F.f32_to_bf16_bits(f))


@pytest.mark.parametrize("shape,bh,bw", [((257, 130), 128, 128), ((64, 200), 1, 128), ((1, 1000), 1, 128),
                                          ((128, 128), 128, 128), ((300, 384), 128, 128)])
def test_block_quantisation_and_inverse_agree(shape, bh, bw):
    R, C = shape
    bits = normal_bf16(3, R, 2, C, R * C, 0.02).reshape(R, C)
    bits[0, :min(C, 8)] = [0x0000, 0x8000, 0x0001, 0x8001, 0x7F7F, 0x3F80, 0xBF80, 0x0080][:min(C, 8)]
    if R > 130:
        bits[128:, :] = 0                               # all-zero blocks
    c1, s1 = F.quantise_matrix(bits, bh, bw)
    c2, s2 = OC.quantise_matrix(bits, bh, bw)
    assert np.array_equal(c1, c2) and np.array_equal(s1.view(np.uint32), s2.view(np.uint32))
    spec = P.TensorSpec(R if R > 1 else C, C if R > 1 else 0, P.BLOCK_128x128 if bh == 128 else P.BLOCK_1x128)
    want = F.dequantise_tensor(c1.reshape(-1), s1.reshape(-1), spec).reshape(R, C)
    assert np.array_equal(OC.dequantise_matrix(c1, s1, bh, bw), want)


def test_pack_and_reduce_agree():
    wl, pl = toy()
    params = gen_params(wl, seed=11)
    assert np.array_equal(OC.ragged_pack(params, pl.offsets, pl.total), D.ragged_pack(params, pl.offsets, pl.total))
    for k in range(pl.m):
        parts = np.stack([gen_partial(wl, 12, w, pl.S) for w in range(wl.world)])
        segs = pl.rank_segments(k)
        a, b = D.shard_reduce(parts, segs), OC.shard_reduce(parts, segs)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


@pytest.mark.parametrize("W", [1, 3, 8, 9, 64, 100])
def test_ordered_mean_and_abs_sum_agree(W):
    """The C statements of the stated-order fp32 mean and of the error scale against the numpy
    ones, bit for bit, on a region with padding between two payload segments."""
    S = 5000
    parts = np.stack([normal_bf16(13, W, 1, w, S, 1e-3) for w in range(W)])
    parts[:, 7] = 0x7F00                        # large magnitudes: cancellation and rounding at work
    parts[W // 2, 7] = 0xFF00
    segs = [(0, 0, 16, 2000), (1, 0, 2500, 2400)]
    a, b = D.shard_reduce_f32_ordered(parts, segs), OC.shard_reduce_f32_ordered(parts, segs)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32))
    assert np.array_equal(D.shard_reduce_abs_sum(parts), OC.shard_reduce_abs_sum(parts))
    x, y = D.shard_reduce(parts, segs), OC.shard_reduce(parts, segs)
    assert np.array_equal(x.view(np.uint32), y.view(np.uint32))


def test_thread_count_does_not_change_results():
    bits = normal_bf16(4, 0, 2, 0, 384 * 512, 0.02).reshape(384, 512)
    default = OC.num_threads()
    try:
        OC.set_num_threads(1)
        one = OC.quantise_matrix(bits, 128, 128)
        OC.set_num_threads(4)
        many = OC.quantise_matrix(bits, 128, 128)
    finally:
        OC.set_num_threads(default)
    assert np.array_equal(one[0], many[0]) and np.array_equal(one[1], many[1])
