"""Pins for the oracle of the DBuffer's group-level add / scale / zero / scaled copy
(Section 5, "Distributed Buffer"): exact rational arithmetic with explicit roundings, the
library's own fp32 / bf16 arithmetic, and algebraic special cases."""
from fractions import Fraction

import numpy as np
import torch

from oracle import dbuffer as D
from oracle import group_ops as G
from oracle import plan as P
from workloads import WORKLOADS, gen_params


def toy():
    wl = WORKLOADS[1]
    specs = [P.TensorSpec(t.rows, t.cols, t.mode) for t in wl.tensors]
    return wl, P.make_plan(specs, wl.world, wl.align_bytes, wl.min_itemsize)


def payload_mask(pl):
    m = np.zeros(pl.total, dtype=bool)
    for s, l in zip(pl.specs, pl.offsets):
        m[l:l + s.e] = True
    return m


def bf16_fraction(bits: int) -> Fraction:
    s, E, M = bits >> 15, (bits >> 7) & 0xFF, bits & 0x7F
    mag = Fraction(M, 128) * Fraction(2) ** -126 if E == 0 else (1 + Fraction(M, 128)) * Fraction(2) ** (E - 127)
    return -mag if s else mag


def round_binary(q: Fraction, precision: int, emin: int = -126) -> Fraction:
    """q rounded to the nearest number with `precision` significant bits (ties to even),
    gradual underflow below 2^emin.  No overflow handling: the test keeps values small."""
    if q == 0:
        return q
    a = abs(q)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    while Fraction(2) ** e > a:
        e -= 1
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    ulp = Fraction(2) ** (max(e, emin) - precision + 1)
    n = a / ulp
    f = n.numerator // n.denominator
    r = n - f
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and f % 2 == 1):
        f += 1
    return f * ulp if q > 0 else -f * ulp


def f32_fraction(x) -> Fraction:
    return Fraction(float(np.float32(x)))


def test_round_binary_helper_on_known_values():
    assert round_binary(Fraction(1, 3), 24) == Fraction(float(np.float32(1.0 / 3.0)))
    assert round_binary(Fraction(1) + Fraction(1, 256), 8) == 1                      # tie -> even
    assert round_binary(Fraction(1) + Fraction(3, 256), 8) == 1 + Fraction(1, 64)    # tie -> even (up)
    assert round_binary(Fraction(2) ** -140, 24) == Fraction(2) ** -140              # fp32 subnormal, exact
    assert round_binary(Fraction(3, 2) * Fraction(2) ** -149, 24) == Fraction(2) ** -148


def test_bf16_rounding_matches_library_cast():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(200000).astype(np.float32) * np.float32(3e-3),
                        np.array([1.00390625, 1.01171875, -1.00390625, 0.0, -0.0, 3.0e-39, 65280.0],
                                 dtype=np.float32)])
    lib = torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(G.f32_to_bf16_bits(x), lib)


def test_scale_and_add_exact_rational_on_sample():
    wl, pl = toy()
    rng = np.random.default_rng(11)
    params = gen_params(wl, seed=3)
    grads = gen_params(wl, seed=4)
    db = D.ragged_pack(params, pl.offsets, pl.total)
    for alpha in (1.0 / 3.0, -0.015625, 0.7310585975646973):
        a = f32_fraction(alpha)
        scaled = G.group_scale(db, pl.offsets, [s.e for s in pl.specs], alpha)
        added = G.group_add(db, grads, pl.offsets, alpha)
        pscaled = G.pack_scaled(grads, pl.offsets, pl.total, alpha)
        for t, (spec, l) in enumerate(zip(pl.specs, pl.offsets)):
            for i in rng.integers(0, spec.e, size=25).tolist() + [0, spec.e - 1]:
                d = bf16_fraction(int(db[l + i]))
                g = bf16_fraction(int(grads[t].reshape(-1)[i]))
                want_scale = round_binary(round_binary(d * a, 24), 8)
                want_add = round_binary(round_binary(d + round_binary(a * g, 24), 24), 8)
                want_ps = round_binary(round_binary(g * a, 24), 8)
                assert bf16_fraction(int(scaled[l + i])) == want_scale
                assert bf16_fraction(int(added[l + i])) == want_add
                assert bf16_fraction(int(pscaled[l + i])) == want_ps


def test_against_library_fp32_arithmetic():
    wl, pl = toy()
    params = gen_params(wl, seed=6)
    grads = gen_params(wl, seed=7)
    db = D.ragged_pack(params, pl.offsets, pl.total)
    gb = D.ragged_pack(grads, pl.offsets, pl.total)
    alpha = 0.25 + 2.0 ** -20
    m = payload_mask(pl)
    tdb = torch.from_numpy(db.view(np.int16)).view(torch.bfloat16).float()
    tgb = torch.from_numpy(gb.view(np.int16)).view(torch.bfloat16).float()
    a = torch.tensor(alpha, dtype=torch.float32)
    lib_scale = (tdb * a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    prod = tgb * a
    lib_add = (tdb + prod).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    got_scale = G.group_scale(db, pl.offsets, [s.e for s in pl.specs], alpha)
    got_add = G.group_add(db, grads, pl.offsets, alpha)
    assert np.array_equal(got_scale[m], lib_scale[m])
    assert np.array_equal(got_add[m], lib_add[m])
    assert np.all(got_scale[~m] == 0) and np.all(got_add[~m] == 0)


def test_algebraic_special_cases():
    wl, pl = toy()
    params = gen_params(wl, seed=8)
    grads = gen_params(wl, seed=9)
    sizes = [s.e for s in pl.specs]
    db = D.ragged_pack(params, pl.offsets, pl.total)
    m = payload_mask(pl)
    # alpha = 1 leaves every bf16 value as it is; powers of two only move the exponent
    assert np.array_equal(G.group_scale(db, pl.offsets, sizes, 1.0), db)
    up = G.group_scale(db, pl.offsets, sizes, 4.0)
    normal = m & ((db & 0x7F80) != 0)
    assert np.array_equal(up[normal], db[normal] + np.uint16(2 << 7))
    # adding into a zeroed buffer with alpha = 1 is the copy; pack_scaled = scale after pack
    zero = G.group_zero(pl.total)
    assert zero.dtype == np.uint16 and zero.size == pl.total and not zero.any()
    packed = D.ragged_pack(grads, pl.offsets, pl.total)
    added = G.group_add(zero, grads, pl.offsets, 1.0)
    nz = (packed & 0x7FFF) != 0                       # x + (+0) keeps x except -0 -> +0
    assert np.array_equal(added[nz], packed[nz]) and np.all((added[~nz] & 0x7FFF) == 0)
    for alpha in (0.5, 1.0 / 64.0, -3.0, 1e-3):
        assert np.array_equal(G.pack_scaled(grads, pl.offsets, pl.total, alpha),
                              G.group_scale(packed, pl.offsets, sizes, alpha))
    # a + (-1) * a = 0 exactly; negative alpha never writes into the padding
    cancel = G.group_add(db, params, pl.offsets, -1.0)
    assert np.all((cancel & 0x7FFF) == 0)
    neg = G.group_scale(db, pl.offsets, sizes, -2.0)
    assert np.all(neg[~m] == 0)
    assert np.array_equal(neg[m] & 0x8000, (db[m] ^ 0x8000) & 0x8000)
