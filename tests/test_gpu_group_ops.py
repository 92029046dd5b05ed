"""GPU parity of the DBuffer's group-level add / scale / zero / scaled copy against the CPU
oracle, bit for bit, through the C ABI: toy and ragged units (odd pitches, element-aligned
plans, element-aligned storage), the config-2 unit at full size, reordered plans, error codes."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import dbuffer as OD
from oracle import group_ops as OG
from paper_2602_22437_amd import binding as B
from workloads import MODE_128x128, MODE_1x128, MODE_WHOLE, WORKLOADS, gen_params, normal_bf16

from gpu_util import Unit, bits_of, say, to_dev_bf16

pytestmark = pytest.mark.gpu

ALPHAS = (1.0 / 64.0, -0.37109375, 1.0, 3.0e-5)
GARBAGE = 0x4300   # bf16 128.0: what padding must never turn into


def first_diff(got, want, what):
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        raise AssertionError(f"{what}: {bad.size} differ, first at {bad[:6]}: got {got[bad[:6]]} want {want[bad[:6]]}")


def check_group_ops(u: Unit, params, grads, label, dev_grads=None):
    sizes = [s.e for s in u.specs]
    base = OD.ragged_pack(params, u.oracle.offsets, u.total)
    dev_g = dev_grads if dev_grads is not None else [to_dev_bf16(g) for g in grads]
    tab = u.table(dev_g)
    for alpha in ALPHAS:
        say(f"pack_scaled {label} alpha={alpha}")
        dbuf = torch.full((u.total,), GARBAGE, dtype=torch.int16, device="cuda").view(torch.bfloat16)
        B.rs_pack_scaled(u.plan, tab, alpha, dbuf)
        torch.cuda.synchronize()
        first_diff(bits_of(dbuf), OG.pack_scaled(grads, u.oracle.offsets, u.total, alpha), f"pack_scaled {label}")

        say(f"group_add {label} alpha={alpha}")
        dbuf = to_dev_bf16(base)
        B.rs_group_add(u.plan, tab, alpha, dbuf)
        torch.cuda.synchronize()
        first_diff(bits_of(dbuf), OG.group_add(base, grads, u.oracle.offsets, alpha), f"group_add {label}")

        say(f"group_scale {label} alpha={alpha}")
        dbuf = to_dev_bf16(base)
        B.rs_group_scale(u.plan, alpha, dbuf)
        torch.cuda.synchronize()
        first_diff(bits_of(dbuf), OG.group_scale(base, u.oracle.offsets, sizes, alpha), f"group_scale {label}")

    # add and scale must not look at or write padding: poison it and see it survive
    pay = np.zeros(u.total, dtype=bool)
    for l, e in zip(u.oracle.offsets, sizes):
        pay[l:l + e] = True
    poisoned = base.copy()
    poisoned[~pay] = GARBAGE
    for name, run, want in (
            ("group_add", lambda d: B.rs_group_add(u.plan, tab, 0.5, d),
             OG.group_add(poisoned, grads, u.oracle.offsets, 0.5)),
            ("group_scale", lambda d: B.rs_group_scale(u.plan, -2.0, d),
             OG.group_scale(poisoned, u.oracle.offsets, sizes, -2.0))):
        say(f"{name} {label} with poisoned padding")
        dbuf = to_dev_bf16(poisoned)
        run(dbuf)
        torch.cuda.synchronize()
        got = bits_of(dbuf)
        first_diff(got, want, f"{name} poisoned {label}")
        assert np.all(got[~pay] == GARBAGE)

    say(f"group_zero {label}")
    dbuf = to_dev_bf16(poisoned)
    B.rs_group_zero(u.plan, dbuf)
    torch.cuda.synchronize()
    first_diff(bits_of(dbuf), OG.group_zero(u.total), f"group_zero {label}")


def test_config1_group_ops():
    wl = WORKLOADS[1]
    u = Unit.from_workload(wl)
    try:
        check_group_ops(u, gen_params(wl, seed=21), gen_params(wl, seed=22), "cfg1")
    finally:
        u.close()


RAGGED = [
    ([(257, 130, MODE_128x128), (5, 0, MODE_1x128), (129, 7, MODE_128x128), (300, 0, MODE_1x128)], 3, 16, 1, 0),
    ([(257, 130, MODE_128x128), (383, 0, MODE_1x128), (129, 8, MODE_128x128)], 4, 16, 1, 1),   # A = 1
    ([(17, 24, MODE_1x128), (250, 0, MODE_1x128), (128, 256, MODE_128x128)], 7, 32, 1, 2),
    ([(128, 128, MODE_128x128)], 8, 16, 1, 0),                                                 # empty ranks
    ([(300, 200, MODE_WHOLE), (64, 64, MODE_WHOLE), (77, 0, MODE_1x128)], 4, 16, 2, 0),        # bf16-only plan
]


@pytest.mark.parametrize("case", range(len(RAGGED)))
def test_ragged_units_group_ops(case):
    tensors, world, align, item, A = RAGGED[case]
    u = Unit(tensors, world, align, item, A)
    try:
        params = [normal_bf16(31, case, 0, i, s.e, 0.02) for i, s in enumerate(u.specs)]
        grads = [normal_bf16(31, case, 1, i, s.e, 1e-3) for i, s in enumerate(u.specs)]
        # tiny and special values: subnormal bf16, -0, values whose product underflows
        grads[0][:6] = np.array([0x0001, 0x8000, 0x0000, 0x807F, 0x0080, 0x7F7F], dtype=np.uint16)
        params[0][:6] = np.array([0x8001, 0x0000, 0x8000, 0x007F, 0x8080, 0x0001], dtype=np.uint16)
        check_group_ops(u, params, grads, f"ragged{case}")
    finally:
        u.close()


def test_element_aligned_storage_group_ops():
    """Gradient tensors that are views at odd element offsets: the per-element path."""
    tensors = [(130, 136, MODE_128x128), (700, 0, MODE_1x128), (64, 256, MODE_1x128)]
    u = Unit(tensors, 3)
    try:
        params = [normal_bf16(32, 0, 0, i, s.e, 0.02) for i, s in enumerate(u.specs)]
        grads = [normal_bf16(32, 0, 1, i, s.e, 1e-3) for i, s in enumerate(u.specs)]
        holders = [torch.zeros(g.size + 8, dtype=torch.bfloat16, device="cuda") for g in grads]
        views = []
        for i, (h, g) in enumerate(zip(holders, grads)):
            v = h[1 + 2 * i:1 + 2 * i + g.size]
            v.copy_(to_dev_bf16(g))
            views.append(v)
        check_group_ops(u, params, grads, "odd-storage", dev_grads=views)
    finally:
        u.close()


def test_reordered_plan_group_ops():
    tensors = [(512, 256, MODE_128x128), (300, 0, MODE_1x128), (128, 384, MODE_128x128), (64, 640, MODE_1x128)]
    u = Unit(tensors, 5, order=B.RS_ORDER_SHAPE)
    try:
        params = [normal_bf16(33, 0, 0, i, s.e, 0.02) for i, s in enumerate(u.specs)]
        grads = [normal_bf16(33, 0, 1, i, s.e, 1e-3) for i, s in enumerate(u.specs)]
        check_group_ops(u, params, grads, "by-shape order")
    finally:
        u.close()


def test_config2_group_ops_full_size():
    """The benched unit (218 M elements, W = 64): accumulate, scale and scaled copy, whole buffer."""
    wl = WORKLOADS[2]
    u = Unit.from_workload(wl)
    try:
        say("config 2: generating parameters and gradients on the host")
        params = gen_params(wl, seed=1)
        grads = gen_params(wl, seed=2)
        sizes = [s.e for s in u.specs]
        base = OD.ragged_pack(params, u.oracle.offsets, u.total)
        tab = u.table([to_dev_bf16(g) for g in grads])
        alpha = 1.0 / 64.0
        say("config 2: pack_scaled")
        dbuf = torch.full((u.total,), GARBAGE, dtype=torch.int16, device="cuda").view(torch.bfloat16)
        B.rs_pack_scaled(u.plan, tab, alpha, dbuf)
        torch.cuda.synchronize()
        first_diff(bits_of(dbuf), OG.pack_scaled(grads, u.oracle.offsets, u.total, alpha), "cfg2 pack_scaled")
        say("config 2: group_add")
        dbuf = to_dev_bf16(base)
        B.rs_group_add(u.plan, tab, alpha, dbuf)
        torch.cuda.synchronize()
        first_diff(bits_of(dbuf), OG.group_add(base, grads, u.oracle.offsets, alpha), "cfg2 group_add")
        say("config 2: group_scale")
        dbuf = to_dev_bf16(base)
        B.rs_group_scale(u.plan, alpha, dbuf)
        torch.cuda.synchronize()
        first_diff(bits_of(dbuf), OG.group_scale(base, u.oracle.offsets, sizes, alpha), "cfg2 group_scale")
        say("config 2: group_zero")
        B.rs_group_zero(u.plan, dbuf)
        torch.cuda.synchronize()
        assert not bits_of(dbuf).any()
    finally:
        u.close()


def test_group_op_argument_errors():
    u = Unit([(256, 128, MODE_128x128)], 2)
    try:
        g = torch.zeros(256 * 128, dtype=torch.bfloat16, device="cuda")
        tab = u.table([g])
        dbuf = torch.zeros(u.total + 8, dtype=torch.bfloat16, device="cuda")
        P = C.c_void_p
        for alpha in (float("nan"), float("inf")):
            assert B.raw_call("rs_group_scale", P(u.plan), C.c_float(alpha), P(dbuf.data_ptr()), P(0)) == B.RS_EINVAL
            assert B.raw_call("rs_group_add", P(u.plan), P(tab), C.c_float(alpha), P(dbuf.data_ptr()), P(0)) == B.RS_EINVAL
        assert B.raw_call("rs_group_scale", P(u.plan), C.c_float(1.0), P(dbuf.data_ptr() + 2), P(0)) == B.RS_EALIGN
        assert B.raw_call("rs_group_zero", P(u.plan), P(dbuf.data_ptr() + 2), P(0)) == B.RS_EALIGN
        assert B.raw_call("rs_group_zero", P(u.plan), P(0), P(0)) == B.RS_EINVAL
        assert B.raw_call("rs_pack_scaled", P(u.plan), P(0), C.c_float(1.0), P(dbuf.data_ptr()), P(0)) == B.RS_EINVAL
        assert B.raw_call("rs_group_add", P(0), P(tab), C.c_float(1.0), P(dbuf.data_ptr()), P(0)) == B.RS_EINVAL
        torch.cuda.synchronize()
        assert not bits_of(dbuf).any()      # no failing call wrote anything
    finally:
        u.close()


@pytest.mark.parametrize("groups,gap", [(1, 0), (3, 0), (2, 24)])
def test_strided_regions_of_a_2d_mesh(groups, gap):
    """A buffer gathered over a (world x groups) device mesh, FSDP rank outermost (the stride
    metadata of StridedRaggedShard, Section 4): `groups` strided unpacks materialise the full
    tensors with no intermediate copy; strided packs are the inverse and leave everything
    between the addressed regions alone."""
    tensors = [(257, 136, MODE_128x128), (300, 0, MODE_1x128), (128, 384, MODE_128x128), (33, 7, MODE_1x128)]
    W = 4
    u = Unit(tensors, W)
    try:
        S = u.S
        stride = groups * S + gap                       # gap: unrelated data between rank rows
        sizes = [s.e for s in u.specs]
        rng = np.random.default_rng(70 + groups)
        gathered = rng.integers(0, 1 << 16, size=W * stride, dtype=np.uint16)
        # bf16 patterns are arbitrary bit patterns here: the copies must keep them bit for bit
        d_gathered = to_dev_bf16(gathered)
        full = [torch.full((groups * e,), 0x7FC0, dtype=torch.int16, device="cuda").view(torch.bfloat16) for e in sizes]
        for g in range(groups):
            say(f"unpack_bf16_strided: group {g} of {groups}, stride {stride}")
            starts = [k * stride + g * S for k in range(W)]
            if gap == 0:
                assert starts == OD.strided_region_starts(W, S, groups, g)
            views = [f[g * e:(g + 1) * e] for f, e in zip(full, sizes)]
            B.rs_unpack_bf16_strided(u.plan, d_gathered[g * S:], stride, u.table(views))
            torch.cuda.synchronize()
            want = OD.unpack_bf16_strided(gathered, u.oracle.offsets, sizes, S, starts)
            for i, (v, w_) in enumerate(zip(views, want)):
                first_diff(bits_of(v), w_, f"strided unpack tensor {i} group {g}")
        # inverse: pack every group's slices into a buffer full of a marker
        marker = np.full(W * stride, 0x4300, dtype=np.uint16)
        d_out = to_dev_bf16(marker)
        want_buf = marker
        host_full = [bits_of(f) for f in full]
        for g in range(groups):
            say(f"pack_strided: group {g} of {groups}")
            starts = [k * stride + g * S for k in range(W)]
            views = [f[g * e:(g + 1) * e] for f, e in zip(full, sizes)]
            B.rs_pack_strided(u.plan, u.table(views), d_out[g * S:], stride)
            torch.cuda.synchronize()
            want_buf = OD.ragged_pack_strided(want_buf, [h[g * e:(g + 1) * e] for h, e in zip(host_full, sizes)],
                                              u.oracle.offsets, S, starts)
            first_diff(bits_of(d_out), want_buf, f"strided pack after group {g}")
        if gap:
            got = bits_of(d_out).reshape(W, stride)
            assert np.all(got[:, groups * S:] == 0x4300)
        P = C.c_void_p
        assert B.raw_call("rs_unpack_bf16_strided", P(u.plan), P(d_gathered.data_ptr()), C.c_int64(S - 8),
                          P(u.tables[0]), P(0)) == B.RS_EINVAL
        assert B.raw_call("rs_pack_strided", P(u.plan), P(u.tables[0]), P(d_out.data_ptr()), C.c_int64(S + 4),
                          P(0)) == B.RS_EALIGN
    finally:
        u.close()


@pytest.mark.parametrize("groups,gap", [(1, 0), (3, 0), (2, 48)])
def test_strided_fp8_unpack_of_a_2d_mesh(groups, gap):
    """rs_unpack_strided / rs_unpack_f32_strided: FP8 codes gathered over a (world x groups) mesh,
    every group with its own scale array; `groups` launches materialise the full tensors in bf16
    and in fp32 with no intermediate copy, bit for bit what the oracle's reshuffle gives."""
    from oracle import fp8 as OF
    tensors = [(257, 136, MODE_128x128), (300, 0, MODE_1x128), (128, 384, MODE_128x128), (33, 8, MODE_1x128)]
    W = 4
    u = Unit(tensors, W)
    try:
        S = u.S
        stride = groups * S + gap
        sizes = [s.e for s in u.specs]
        nb = u.oracle.scale_bases()[-1]
        rng = np.random.default_rng(80 + groups)
        gathered = rng.integers(0, 0x7F, size=W * stride, dtype=np.uint8) | (
            rng.integers(0, 2, size=W * stride, dtype=np.uint8) << 7)
        d_codes = torch.from_numpy(gathered).cuda()
        full16 = [torch.full((groups * e,), 0x7FC0, dtype=torch.int16, device="cuda").view(torch.bfloat16) for e in sizes]
        full32 = [torch.full((groups * e,), float("nan"), dtype=torch.float32, device="cuda") for e in sizes]
        for g in range(groups):
            scales = (rng.random(nb).astype(np.float32) + np.float32(0.25)) * np.float32(2e-3)
            d_scales = torch.from_numpy(scales).cuda()
            starts = [k * stride + g * S for k in range(W)]
            say(f"unpack_strided: group {g} of {groups}, stride {stride}")
            v16 = [f[g * e:(g + 1) * e] for f, e in zip(full16, sizes)]
            v32 = [f[g * e:(g + 1) * e] for f, e in zip(full32, sizes)]
            B.rs_unpack_strided(u.plan, d_codes[g * S:], stride, d_scales, u.table(v16))
            B.rs_unpack_f32_strided(u.plan, d_codes[g * S:], stride, d_scales, u.table(v32))
            torch.cuda.synchronize()
            want16 = OF.dequant_unpack_strided(u.oracle, gathered, starts, scales)
            want32 = OF.dequant_unpack_strided(u.oracle, gathered, starts, scales, f32=True)
            for i in range(len(sizes)):
                first_diff(bits_of(v16[i]), want16[i], f"strided fp8 unpack tensor {i} group {g}")
                assert np.array_equal(v32[i].cpu().numpy().view(np.uint32), want32[i].view(np.uint32)), (i, g)
        P = C.c_void_p
        tab = u.tables[0]
        sc = torch.zeros(nb, dtype=torch.float32, device="cuda")
        assert B.raw_call("rs_unpack_strided", P(u.plan), P(d_codes.data_ptr()), C.c_int64(S - 16), P(sc.data_ptr()),
                          P(tab), P(0)) == B.RS_EINVAL
        assert B.raw_call("rs_unpack_f32_strided", P(u.plan), P(d_codes.data_ptr()), C.c_int64(S + 4), P(sc.data_ptr()),
                          P(tab), P(0)) == B.RS_EALIGN
    finally:
        u.close()


@pytest.mark.parametrize("seed", range(12))
def test_random_units_group_ops(seed):
    """Random units (any block mode, odd pitches, element-aligned starts, reordered buffers)."""
    import random
    rnd = random.Random(7000 + seed)
    n = rnd.randint(1, 7)
    tensors = []
    for _ in range(n):
        kind = rnd.random()
        if kind < 0.3:
            tensors.append((rnd.randint(1, 3000), 0, MODE_1x128))
        elif kind < 0.6:
            tensors.append((rnd.randint(1, 400), rnd.choice([8, 24, 30, 128, 130, 136, 256, 1100]), MODE_128x128))
        elif kind < 0.8:
            tensors.append((rnd.randint(1, 60), rnd.choice([8, 40, 128, 333]), MODE_1x128))
        else:
            tensors.append((rnd.randint(1, 80), rnd.randint(1, 90), MODE_WHOLE))
    world = rnd.choice([1, 2, 3, 5, 8, 16])
    align, item = rnd.choice([(16, 1), (16, 2), (32, 2)])
    A = rnd.choice([0, 0, 1, 4])
    if A and (align // item) % A:
        A = 0
    u = Unit(tensors, world, align, item, A, order=rnd.choice([0, 1, 2, 3]))
    try:
        say(f"random unit {seed}: {tensors} W={world} align={align}/{item} A={A}")
        params = [normal_bf16(32, seed, 0, i, s.e, 0.02) for i, s in enumerate(u.specs)]
        grads = [normal_bf16(32, seed, 1, i, s.e, 1e-3) for i, s in enumerate(u.specs)]
        check_group_ops(u, params, grads, f"random{seed}")
    finally:
        u.close()
