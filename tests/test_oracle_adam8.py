"""Pins for the oracle of the block-wise 8-bit optimiser state and the Adam step on a ragged
shard (Section 6.3): hand-stated codec values, exact rational arithmetic with explicit
roundings, torch's AdamW as the library special case, block ownership by brute force, and
"a rank's step from its own region equals the whole-tensor step"."""
from fractions import Fraction
from math import isqrt

import numpy as np
import pytest
import torch

from oracle import adam8 as A
from oracle import plan as P

F = np.float32


# ---------------------------------------------------------------------------------------------
# codec
# ---------------------------------------------------------------------------------------------

def test_codec_hand_values_and_ties():
    # absmax 127 makes the step exactly 1: codes are rint of the values, ties to even
    x = np.zeros((32, 32), dtype=np.float32)
    vals = [127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, -126.5, 3.49, -3.51]
    x[0, :len(vals)] = vals
    codes, amax = A.quantise_state(x, False, True)
    assert amax.tolist() == [127.0]
    assert codes[0, :len(vals)].tolist() == [127, 0, 2, 2, 0, -2, -2, 126, -126, 3, -4]
    assert A.dequantise_state(codes, amax, False, True)[0, :4].tolist() == [127.0, 0.0, 2.0, 2.0]
    # second moment: absmax 255, step 1, codes 0..255
    v = np.zeros((32, 32), dtype=np.float32)
    vv = [255.0, 0.5, 1.5, 254.5, 253.5, 100.25]
    v[3, :len(vv)] = vv
    codes, amax = A.quantise_state(v, False, False)
    assert amax.tolist() == [255.0] and codes[3, :len(vv)].tolist() == [255, 0, 2, 254, 254, 100]


def test_codec_blocks_are_32x32_tiles_and_128_runs():
    x = np.zeros((70, 40), dtype=np.float32)
    x[0, 0], x[31, 31], x[32, 0], x[69, 39], x[5, 33] = 1, -2, 3, -4, 5
    _, amax = A.quantise_state(x, False, True)
    # grid 3 x 2: (0,0) holds 1 and -2, (0,1) holds 5, (1,0) holds 3, (2,1) holds -4
    assert amax.tolist() == [2, 5, 3, 0, 0, 4]
    y = np.zeros((1, 300), dtype=np.float32)
    y[0, 127], y[0, 128], y[0, 299] = 7, 8, 9
    _, amax = A.quantise_state(y, True, False)
    assert amax.tolist() == [7, 8, 9]


def test_codec_extremes_zero_blocks_and_error_bound():
    rng = np.random.default_rng(3)
    x = (rng.standard_normal((96, 64)) * 1e-3).astype(np.float32)
    x[32:64, 0:32] = 0
    for signed in (True, False):
        src = x if signed else x * x
        codes, amax = A.quantise_state(src, False, signed)
        top = 127 if signed else 255
        back = A.dequantise_state(codes, amax, False, signed)
        for b, rs, cs in A._blocks(96, 64, False):
            blk, c = src[rs, cs], codes[rs, cs]
            if amax[b] == 0:
                assert not c.any() and not back[rs, cs].any()
                continue
            assert np.abs(c).max() == top                   # the absmax element takes the last code
            assert c.min() >= (-top if signed else 0)
            step = float(amax[b]) / top
            assert np.all(np.abs(back[rs, cs].astype(np.float64) - blk) <= step * (0.5 + 1e-5))
    assert np.count_nonzero(amax == 0) == 1


# ---------------------------------------------------------------------------------------------
# the fp32 update: exact rationals, and torch.optim.AdamW as an independent formula
# ---------------------------------------------------------------------------------------------

def rnd(q: Fraction, precision: int = 24, emin: int = -126) -> Fraction:
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


def sqrt_rnd(q: Fraction) -> Fraction:
    """Correctly rounded fp32 square root of a non-negative rational (normal results)."""
    if q == 0:
        return q
    e = 0
    while Fraction(4) ** e > q:
        e -= 1
    while Fraction(4) ** (e + 1) <= q:
        e += 1                                   # sqrt(q) in [2^e, 2^(e+1))
    ulp = Fraction(2) ** (e - 23)
    n = q / (ulp * ulp)                          # (sqrt(q) / ulp)^2
    f = isqrt(n.numerator // n.denominator)      # floor(sqrt(q) / ulp)
    half = Fraction(f) * f + f + Fraction(1, 4)  # (f + 1/2)^2
    if n > half or (n == half and f % 2 == 1):
        f += 1
    return f * ulp


def fr(x) -> Fraction:
    return Fraction(float(F(x)))


def test_sqrt_helper():
    for x in (2.0, 3.0, 1e-7, 0.30000001192092896, 16.0, 1.0000001192092896):
        assert sqrt_rnd(fr(x)) == Fraction(float(np.sqrt(F(x))))


def test_update_exact_rational_on_sample():
    rng = np.random.default_rng(17)
    n = 60
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    w = (rng.standard_normal(n) * 0.02).astype(np.float32)
    m0 = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    v0 = (rng.standard_normal(n) ** 2 * 1e-6).astype(np.float32)
    g[0], m0[1], v0[2] = 0, 0, 0
    h = A.Hyper(lr=3e-4, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=7)
    m, v, w2 = A.adam_update(g, w, m0, v0, h)
    b1, b2, eps = fr(0.9), fr(0.95), fr(1e-8)
    omb1, omb2 = fr(1.0 - 0.9), fr(1.0 - 0.95)
    bc1, bc2 = 1.0 - 0.9 ** 7, 1.0 - 0.95 ** 7
    step_size, bc2s, decay = fr(3e-4 / bc1), fr(bc2 ** 0.5), fr(1.0 - 3e-4 * 0.1)
    for i in range(n):
        gi, wi, mi, vi = fr(g[i]), fr(w[i]), fr(m0[i]), fr(v0[i])
        em = rnd(rnd(b1 * mi) + rnd(omb1 * gi))
        ev = rnd(rnd(b2 * vi) + rnd(omb2 * rnd(gi * gi)))
        denom = rnd(rnd(sqrt_rnd(ev) / bc2s) + eps)
        ew = rnd(rnd(wi * decay) - rnd(step_size * rnd(em / denom)))
        assert fr(m[i]) == em and fr(v[i]) == ev and fr(w2[i]) == ew, i


@pytest.mark.parametrize("step", [1, 2, 50])
def test_update_matches_torch_adamw(step):
    rng = np.random.default_rng(23)
    n = 4096
    g = (rng.standard_normal(n) * 1e-3).astype(np.float32)
    w = (rng.standard_normal(n) * 0.02).astype(np.float32)
    m0 = np.zeros(n, np.float32) if step == 1 else (rng.standard_normal(n) * 1e-3).astype(np.float32)
    v0 = np.zeros(n, np.float32) if step == 1 else (rng.standard_normal(n) ** 2 * 1e-6).astype(np.float32)
    h = A.Hyper(lr=1e-3, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01, step=step)
    m, v, w2 = A.adam_update(g, w, m0, v0, h)
    p = torch.nn.Parameter(torch.from_numpy(w.copy()))
    opt = torch.optim.AdamW([p], lr=h.lr, betas=(h.beta1, h.beta2), eps=h.eps, weight_decay=h.weight_decay,
                            foreach=False, fused=False, capturable=False, amsgrad=False)
    p.grad = torch.from_numpy(g.copy())
    if step > 1:
        opt.state[p] = {"step": torch.tensor(float(step - 1)), "exp_avg": torch.from_numpy(m0.copy()),
                        "exp_avg_sq": torch.from_numpy(v0.copy())}
    opt.step()
    st = opt.state[p]
    assert np.allclose(st["exp_avg"].numpy(), m, rtol=2e-6, atol=1e-9)   # lerp form: other roundings
    assert np.allclose(st["exp_avg_sq"].numpy(), v, rtol=2e-6, atol=1e-15)
    # the update is at most lr per element; the two formulations differ by a few ulps of it
    assert np.max(np.abs(p.detach().numpy() - w2)) <= 1e-5 * h.lr + 2.0 ** -24 * np.abs(w).max()
    assert np.max(np.abs(w2 - w)) > 0.1 * h.lr             # the step is not a no-op


def test_direction_and_decay_special_cases():
    n = 1024
    w = np.full(n, 0.5, np.float32)
    zero = np.zeros(n, np.float32)
    # no gradient, no state: only the decoupled decay acts
    h = A.Hyper(lr=0.1, beta1=0.9, beta2=0.99, eps=1e-8, weight_decay=0.5, step=1)
    m, v, w2 = A.adam_update(zero, w, zero, zero, h)
    assert not m.any() and not v.any() and np.all(w2 == F(0.5) * (F(1) - F(0.1) * F(0.5)))
    # first step with a constant gradient moves every weight by lr against its sign
    h = A.Hyper(lr=0.01, beta1=0.9, beta2=0.99, eps=1e-12, weight_decay=0.0, step=1)
    g = np.where(np.arange(n) % 2 == 0, 3e-3, -3e-3).astype(np.float32)
    _, _, w2 = A.adam_update(g, w, zero, zero, h)
    assert np.allclose(w2 - w, -0.01 * np.sign(g), rtol=1e-4)


# ---------------------------------------------------------------------------------------------
# layout: which rank owns which state blocks, and shard-local == whole-tensor
# ---------------------------------------------------------------------------------------------

UNITS = [
    ([(256, 384, P.BLOCK_32x32), (384, 0, P.BLOCK_32x32), (96, 64, P.BLOCK_32x32), (70, 40, P.BLOCK_32x32),
      (1000, 0, P.BLOCK_32x32)], 4),
    ([(256, 128, P.BLOCK_128x128), (300, 0, P.BLOCK_1x128), (257, 130, P.BLOCK_128x128)], 3),
    ([(64, 64, P.BLOCK_32x32)], 5),
    ([(40, 200, P.BLOCK_1x128), (128, 256, P.BLOCK_128x128), (33, 136, P.BLOCK_1x128), (500, 0, P.BLOCK_1x128)], 3),
]


def make(unit):
    tensors, world = unit
    specs = [P.TensorSpec(*t) for t in tensors]
    return specs, P.make_plan(specs, world, 16, 1)


@pytest.mark.parametrize("unit", UNITS)
def test_state_ranges_by_brute_force_ownership(unit):
    specs, pl = make(unit)
    bases = A.state_bases(pl)
    owner_of_block = {}
    for t, (s, l) in enumerate(zip(specs, pl.offsets)):
        R, C, one_d = (1, s.rows, True) if s.cols == 0 else (s.rows, s.cols, A.state_runs(s))
        for b, rs, cs in A._blocks(R, C, one_d):
            owners = set()
            for r in range(rs.start, rs.stop):
                for c in (cs.start, cs.stop - 1):
                    owners.add((l + r * C + c) // pl.S)
            assert len(owners) == 1, "a state block is split across ranks"
            owner_of_block[bases[t] + b] = owners.pop()
    assert sorted(owner_of_block) == list(range(bases[-1]))
    for k in range(pl.m):
        lo, hi = A.state_range(pl, k)
        assert [b for b in range(bases[-1]) if owner_of_block[b] == k] == list(range(lo, hi))


def test_unsupported_granularity_is_refused():
    for spec in (P.TensorSpec(64, 256, P.BLOCK_WHOLE), P.TensorSpec(640, 0, P.BLOCK_EXPLICIT, 128)):
        with pytest.raises(ValueError):
            A.state_grid(spec)


def test_row_runs_are_blocks_of_one_row():
    y = np.zeros((3, 300), dtype=np.float32)
    y[0, 127], y[0, 128], y[1, 299], y[2, 0] = 7, 8, 9, -3
    _, amax = A.quantise_state(y, True, True)
    assert amax.tolist() == [7, 8, 0, 0, 0, 9, 3, 0, 0]
    assert A.state_grid(P.TensorSpec(3, 300, P.BLOCK_1x128)) == (3, 3)


@pytest.mark.parametrize("unit", UNITS)
def test_rank_local_step_equals_whole_tensor_step(unit):
    specs, pl = make(unit)
    rng = np.random.default_rng(31)
    h = A.Hyper(lr=2e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=3)
    bases = A.state_bases(pl)
    tot = pl.total
    G, W = np.zeros(tot, np.float32), np.zeros(tot, np.float32)
    MC, VC = np.zeros(tot, np.int8), np.zeros(tot, np.uint8)
    AM, AV = np.zeros(bases[-1], np.float32), np.zeros(bases[-1], np.float32)
    want = dict(W=W.copy(), Pb=np.zeros(tot, np.uint16), MC=MC.copy(), VC=VC.copy(), AM=AM.copy(), AV=AV.copy())
    for t, (s, l) in enumerate(zip(specs, pl.offsets)):
        R, C, one_d = (1, s.rows, True) if s.cols == 0 else (s.rows, s.cols, A.state_runs(s))
        g = (rng.standard_normal((R, C)) * 1e-3).astype(np.float32)
        w = (rng.standard_normal((R, C)) * 0.02).astype(np.float32)
        mc, am = A.quantise_state((rng.standard_normal((R, C)) * 1e-3).astype(np.float32), one_d, True)
        vc, av = A.quantise_state((rng.standard_normal((R, C)) ** 2 * 1e-6).astype(np.float32), one_d, False)
        sl, bs = slice(l, l + s.e), slice(bases[t], bases[t] + am.size)
        G[sl], W[sl], MC[sl], VC[sl] = g.reshape(-1), w.reshape(-1), mc.reshape(-1), vc.reshape(-1)
        AM[bs], AV[bs] = am, av
        res = A.adam8_step_matrix(g, w, mc, vc, am, av, one_d, h)
        want["W"][sl], want["Pb"][sl] = res[0].reshape(-1), res[1].reshape(-1)
        want["MC"][sl], want["VC"][sl] = res[2].reshape(-1), res[3].reshape(-1)
        want["AM"][bs], want["AV"][bs] = res[4], res[5]
    for k in range(pl.m):
        r = slice(k * pl.S, (k + 1) * pl.S)
        lo, hi = A.state_range(pl, k)
        w2, pb, mc2, vc2, am2, av2 = A.adam8_step_shard(pl, k, G[r], W[r], np.zeros(pl.S, np.uint16), MC[r], VC[r],
                                                        AM[lo:hi], AV[lo:hi], h)
        assert np.array_equal(w2, want["W"][r]) and np.array_equal(pb, want["Pb"][r])
        assert np.array_equal(mc2, want["MC"][r]) and np.array_equal(vc2, want["VC"][r])
        assert np.array_equal(am2, want["AM"][lo:hi]) and np.array_equal(av2, want["AV"][lo:hi])


@pytest.mark.parametrize("unit", UNITS)
def test_rank_local_codec_equals_whole_tensor_codec_and_inverts_within_half_a_step(unit):
    specs, pl = make(unit)
    rng = np.random.default_rng(37)
    bases = A.state_bases(pl)
    X = np.zeros(pl.total, np.float32)
    want_c, want_a = np.zeros(pl.total, np.int16), np.zeros(bases[-1], np.float32)
    for t, (s, l) in enumerate(zip(specs, pl.offsets)):
        R, C, runs = (1, s.rows, True) if s.cols == 0 else (s.rows, s.cols, A.state_runs(s))
        x = (rng.standard_normal((R, C)) * 1e-3).astype(np.float32)
        X[l:l + s.e] = x.reshape(-1)
        c, a = A.quantise_state(x, runs, True)
        want_c[l:l + s.e], want_a[bases[t]:bases[t] + a.size] = c.reshape(-1), a
    for k in range(pl.m):
        r = slice(k * pl.S, (k + 1) * pl.S)
        lo, hi = A.state_range(pl, k)
        pad = np.full(pl.S, 0x55, np.int8)
        codes, amax = A.quantise_shard(pl, k, X[r], pad, True)
        pay = np.zeros(pl.S, dtype=bool)
        for _, _, d, n in pl.rank_segments(k):
            pay[d:d + n] = True
        assert np.array_equal(codes[pay], want_c[r][pay].astype(np.int8)) and np.all(codes[~pay] == 0x55)
        assert np.array_equal(amax, want_a[lo:hi])
        back = A.dequantise_shard(pl, k, codes, amax, np.full(pl.S, 9.0, np.float32), True)
        assert np.all(back[~pay] == 9.0)
        # every element within half a quantisation step of its block
        step = np.zeros(pl.S)
        cur = 0
        for dst, n, R, C, runs, nblk in A._segments(pl, k):
            st = np.zeros((R, C))
            for b, rs, cs in A._blocks(R, C, runs):
                st[rs, cs] = float(amax[cur + b]) / 127
            step[dst:dst + n] = st.reshape(-1)
            cur += nblk
        assert np.all(np.abs(back[pay].astype(np.float64) - X[r][pay]) <= step[pay] * (0.5 + 1e-5))
