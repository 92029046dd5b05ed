"""GPU parity of rs_adam8_step (AdamW on the local shard with block-wise 8-bit moments,
Section 6.3) against the CPU oracle, bit for bit on every output (master weights, bf16
parameters, both code arrays, both absmax arrays), through the C ABI, over several consecutive
steps so that the quantised state feeds back."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import adam8 as OA
from paper_2602_22437_amd import binding as B
from workloads import MODE_128x128, MODE_1x128, MODE_32x32, MODE_WHOLE, WORKLOADS

from gpu_util import Unit, say

pytestmark = pytest.mark.gpu

W_SENTINEL, P_SENTINEL, M_SENTINEL, V_SENTINEL = np.float32(123.0), np.uint16(0x4300), np.int8(0x55), np.uint8(0xAA)


def diff(got, want, what):
    if not np.array_equal(got, want):
        bad = np.flatnonzero(got != want)
        raise AssertionError(f"{what}: {bad.size} differ, first at {bad[:6]}: got {got[bad[:6]]} want {want[bad[:6]]}")


def run_steps(u: Unit, rank: int, seed: int, hypers, label, grad_sigma=1e-3, with_param=True, wild=False):
    """Zero state, then one step per entry of `hypers`, each compared with the oracle."""
    S = u.S
    rng = np.random.default_rng(seed)
    pay = np.zeros(S, dtype=bool)
    for _, _, d, n in u.oracle.rank_segments(rank):
        pay[d:d + n] = True
    lo, hi = OA.state_range(u.oracle, rank)
    assert B.rs_plan_state_range(u.plan, rank) == (lo, hi)
    nb = hi - lo
    w = (rng.standard_normal(S) * 0.02).astype(np.float32)
    w[~pay] = W_SENTINEL
    pb = np.full(S, P_SENTINEL, np.uint16)
    mc = np.zeros(S, np.int8)
    vc = np.zeros(S, np.uint8)
    mc[~pay], vc[~pay] = M_SENTINEL, V_SENTINEL
    am, av = np.zeros(nb, np.float32), np.zeros(nb, np.float32)
    d_w = torch.from_numpy(w).cuda()
    d_p = torch.from_numpy(pb.view(np.int16)).cuda()
    d_mc, d_vc = torch.from_numpy(mc).cuda(), torch.from_numpy(vc).cuda()
    d_am = torch.from_numpy(np.concatenate([am, [7.0]]).astype(np.float32)).cuda()   # one guard word behind
    d_av = torch.from_numpy(np.concatenate([av, [7.0]]).astype(np.float32)).cuda()
    for i, h in enumerate(hypers):
        g = (rng.standard_normal(S) * grad_sigma).astype(np.float32)
        if i == 1:
            g[pay & (rng.random(S) < 0.01)] = 0.0
        if wild:       # magnitudes from 1e-30 to 1e+15 side by side: tiny, subnormal and huge second moments
            g = (g * np.float32(1e3) * (np.float32(10.0) ** rng.integers(-30, 16, size=S).astype(np.float32))).astype(np.float32)
        g[~pay] = np.nan                                  # the kernel must not look at padding
        say(f"adam8 {label}: rank={rank} step={h.step} S={S} blocks={nb}")
        B.rs_adam8_step(u.plan, rank, (h.lr, h.beta1, h.beta2, h.eps, h.weight_decay, h.step),
                        torch.from_numpy(g).cuda(), d_w, d_p if with_param else None, d_mc, d_vc, d_am, d_av)
        torch.cuda.synchronize()
        w, pb_new, mc, vc, am, av = OA.adam8_step_shard(u.oracle, rank, g, w, pb, mc, vc, am, av, h)
        if with_param:
            pb = pb_new
        diff(d_w.cpu().numpy().view(np.uint32), w.view(np.uint32), f"master {label} step {h.step}")
        diff(d_p.cpu().numpy().view(np.uint16), pb, f"param {label} step {h.step}")
        diff(d_am.cpu().numpy()[:nb].view(np.uint32), am.view(np.uint32), f"m absmax {label} step {h.step}")
        diff(d_av.cpu().numpy()[:nb].view(np.uint32), av.view(np.uint32), f"v absmax {label} step {h.step}")
        diff(d_mc.cpu().numpy(), mc, f"m codes {label} step {h.step}")
        diff(d_vc.cpu().numpy(), vc, f"v codes {label} step {h.step}")
        assert d_am.cpu().numpy()[nb] == 7.0 and d_av.cpu().numpy()[nb] == 7.0
    # padding untouched in every array
    assert np.all(w[~pay] == W_SENTINEL) and np.all(mc[~pay] == M_SENTINEL) and np.all(vc[~pay] == V_SENTINEL)
    if nb and not wild:
        assert am.max() > 0 and av.max() > 0 and np.abs(mc[pay]).max() == 127 and vc[pay].max() == 255


def hypers(n, lr=2e-3, wd=0.1):
    return [OA.Hyper(lr=lr, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=wd, step=s) for s in range(1, n + 1)]


UNITS = [
    # 32-row granularity (the paper's 8-bit Adam set-up): full and partial tiles, several column strips
    ([(256, 384, MODE_32x32), (384, 0, MODE_32x32), (96, 64, MODE_32x32), (70, 40, MODE_32x32),
      (1000, 0, MODE_32x32)], 4, 0),
    # 128-row granularity shared with FP8 blocks, 1-D tensors in 1x128 mode, odd pitches (130, 30)
    ([(256, 128, MODE_128x128), (300, 0, MODE_1x128), (257, 130, MODE_128x128), (33, 30, MODE_128x128)], 3, 0),
    # element-aligned tensor starts (A = 1) and a pitch that is not a multiple of 4: scalar path
    ([(64, 36, MODE_32x32), (100, 0, MODE_32x32), (37, 35, MODE_32x32)], 3, 1),
    ([(64, 64, MODE_32x32)], 5, 0),                      # most ranks empty
    ([(64, 1100, MODE_32x32), (16384, 0, MODE_32x32)], 2, 0),   # 5 column strips, the last partial; many runs
    # matrices of one-row granularity: runs of 128 along each row, back to back (256) or with a short last run
    ([(40, 200, MODE_1x128), (128, 256, MODE_128x128), (33, 136, MODE_1x128), (70, 256, MODE_1x128), (500, 0, MODE_1x128)], 3, 0),
    ([(19, 130, MODE_1x128), (7, 33, MODE_1x128)], 2, 1),       # A = 1, pitch not a multiple of 4
]


@pytest.mark.parametrize("case", range(len(UNITS)))
def test_adam8_units_every_rank(case):
    tensors, world, A = UNITS[case]
    u = Unit(tensors, world, 16, 1, A)
    try:
        assert B.rs_plan_num_state_blocks(u.plan) == OA.state_bases(u.oracle)[-1]
        assert B.rs_plan_state_bases(u.plan) == OA.state_bases(u.oracle)
        for k in range(world):
            run_steps(u, k, 100 * case + k, hypers(3), f"unit{case}")
    finally:
        u.close()


@pytest.mark.parametrize("case", [0, 1, 5])
def test_adam8_gradients_of_wildly_different_magnitudes(case):
    """Gradients from 1e-30 to 1e+15 in one shard: second moments that are zero, subnormal, tiny and
    huge, quotients far below one code step - every output still bit for bit the oracle's."""
    tensors, world, A = UNITS[case]
    u = Unit(tensors, world, 16, 1, A)
    try:
        for k in range(world):
            run_steps(u, k, 4000 + 10 * case + k, hypers(3), f"wild{case}", wild=True)
    finally:
        u.close()


def test_adam8_without_param_output_and_no_decay():
    u = Unit(UNITS[0][0], UNITS[0][1])
    try:
        run_steps(u, 1, 77, hypers(2, lr=1e-3, wd=0.0), "no-param", with_param=False)
    finally:
        u.close()


def test_adam8_llama_layer_shard_at_32_row_granularity():
    """Config-2 shapes with the 32-row granularity of the paper's 8-bit Adam runs, FSDP size 64:
    a full-size shard (the launch shape the bench times)."""
    wl = WORKLOADS[2]
    tensors = [(t.rows, t.cols, MODE_32x32) for t in wl.tensors]
    u = Unit(tensors, wl.world, wl.align_bytes, wl.min_itemsize)
    try:
        for k in (0, 37):
            run_steps(u, k, 500 + k, hypers(2, lr=3e-4), "llama-32row")
    finally:
        u.close()


def test_adam8_on_the_fp8_plan_of_config2():
    """The same optimiser step on the 128x128 FP8 plan of config 2 (32x32 state tiles nest in it)."""
    u = Unit.from_workload(WORKLOADS[2])
    try:
        run_steps(u, 63, 900, hypers(2, lr=3e-4), "cfg2-fp8-plan")
    finally:
        u.close()


def test_adam8_errors():
    P = C.c_void_p
    u = Unit([(64, 64, MODE_32x32)], 2)
    un = Unit([(64, 64, MODE_WHOLE)], 2, 16, 2)
    try:
        S = u.S
        g = torch.zeros(S + 4, dtype=torch.float32, device="cuda")
        w = torch.zeros(S + 4, dtype=torch.float32, device="cuda")
        p = torch.zeros(S + 8, dtype=torch.bfloat16, device="cuda")
        mc = torch.zeros(S + 16, dtype=torch.int8, device="cuda")
        vc = torch.zeros(S + 16, dtype=torch.uint8, device="cuda")
        am = torch.zeros(8, dtype=torch.float32, device="cuda")
        av = torch.zeros(8, dtype=torch.float32, device="cuda")

        def call(plan, rank, h, gp=None, wp=None):
            hs = B.rs_adam8_hyper(*h)
            return B.raw_call("rs_adam8_step", P(plan), C.c_int(rank), C.byref(hs), P(gp or g.data_ptr()),
                              P(wp or w.data_ptr()), P(p.data_ptr()), P(mc.data_ptr()), P(vc.data_ptr()),
                              P(am.data_ptr()), P(av.data_ptr()), P(0))

        ok = (1e-3, 0.9, 0.95, 1e-8, 0.0, 1)
        assert call(u.plan, 0, ok) == B.RS_OK
        assert call(u.plan, 2, ok) == B.RS_EINVAL
        assert call(u.plan, 0, (1e-3, 1.0, 0.95, 1e-8, 0.0, 1)) == B.RS_EINVAL
        assert call(u.plan, 0, (1e-3, 0.9, -0.1, 1e-8, 0.0, 1)) == B.RS_EINVAL
        assert call(u.plan, 0, (1e-3, 0.9, 0.95, 0.0, 0.0, 1)) == B.RS_EINVAL
        assert call(u.plan, 0, (1e-3, 0.9, 0.95, 1e-8, 0.0, 0)) == B.RS_EINVAL
        assert call(u.plan, 0, (float("nan"), 0.9, 0.95, 1e-8, 0.0, 1)) == B.RS_EINVAL
        assert call(u.plan, 0, ok, gp=g.data_ptr() + 4) == B.RS_EALIGN
        assert call(u.plan, 0, ok, wp=w.data_ptr() + 8) == B.RS_EALIGN
        assert call(un.plan, 0, ok) == B.RS_EUNSUPPORTED
        assert B.raw_call("rs_plan_num_state_blocks", P(un.plan)) == B.RS_EUNSUPPORTED
        torch.cuda.synchronize()
    finally:
        u.close()
        un.close()


def test_adam8_step_batch_equals_per_unit_steps():
    """One launch over rank 1's shard of five units == five rs_adam8_step calls, bit for bit; unit 0
    is also held against the oracle."""
    tensors, world, _ = UNITS[0]
    u = Unit(tensors, world)
    try:
        S, rank, count = u.S, 1, 5
        lo, hi = B.rs_plan_state_range(u.plan, rank)
        nb = hi - lo
        rng = np.random.default_rng(4242)
        h1, h2 = hypers(2)

        def fresh():
            return dict(
                g=[torch.from_numpy((rng.standard_normal(S) * 1e-3).astype(np.float32)).cuda() for _ in range(count)],
                w=[torch.from_numpy((rng.standard_normal(S) * 0.02).astype(np.float32)).cuda() for _ in range(count)],
                p=[torch.zeros(S, dtype=torch.bfloat16, device="cuda") for _ in range(count)],
                mc=[torch.zeros(S, dtype=torch.int8, device="cuda") for _ in range(count)],
                vc=[torch.zeros(S, dtype=torch.uint8, device="cuda") for _ in range(count)],
                am=[torch.zeros(nb, dtype=torch.float32, device="cuda") for _ in range(count)],
                av=[torch.zeros(nb, dtype=torch.float32, device="cuda") for _ in range(count)])
        a = fresh()
        b = {k: [t.clone() for t in v] for k, v in a.items()}
        host = {k: [t.cpu().numpy().copy() for t in v] for k, v in a.items() if k != "p"}
        batch = B.rs_adam8_batch_create(u.plan, rank, a["g"], a["w"], a["p"], a["mc"], a["vc"], a["am"], a["av"])
        for h in (h1, h2):
            tup = (h.lr, h.beta1, h.beta2, h.eps, h.weight_decay, h.step)
            say(f"adam8 batch of {count} units, step {h.step}")
            B.rs_adam8_step_batch(u.plan, batch, tup)
            for i in range(count):
                B.rs_adam8_step(u.plan, rank, tup, b["g"][i], b["w"][i], b["p"][i], b["mc"][i], b["vc"][i],
                                b["am"][i], b["av"][i])
            torch.cuda.synchronize()
            for k in ("w", "p", "mc", "vc", "am", "av"):
                for i in range(count):
                    x, y = a[k][i], b[k][i]
                    if x.dtype == torch.bfloat16:
                        x, y = x.view(torch.int16), y.view(torch.int16)
                    assert torch.equal(x, y), f"{k} of unit {i} differs at step {h.step}"
        B.rs_adam8_batch_destroy(batch)
        # unit 0 against the oracle, two steps from the zero state
        w, pb, mc, vc = host["w"][0], np.zeros(S, np.uint16), host["mc"][0], host["vc"][0].astype(np.uint8)
        am, av = host["am"][0], host["av"][0]
        for h in (h1, h2):
            w, pb, mc, vc, am, av = OA.adam8_step_shard(u.oracle, rank, host["g"][0], w, pb, mc, vc, am, av, h)
        pay = np.zeros(S, dtype=bool)
        for _, _, d, n in u.oracle.rank_segments(rank):
            pay[d:d + n] = True
        diff(a["w"][0].cpu().numpy()[pay].view(np.uint32), w[pay].view(np.uint32), "batch master vs oracle")
        diff(a["mc"][0].cpu().numpy()[pay], mc[pay], "batch m codes vs oracle")
        diff(a["vc"][0].cpu().numpy()[pay], vc[pay], "batch v codes vs oracle")
        diff(a["am"][0].cpu().numpy().view(np.uint32), am.view(np.uint32), "batch m absmax vs oracle")
    finally:
        u.close()


def test_adam8_gpt_oss_shard_with_partial_column_strips():
    """Rank 0's shard of the GPT-OSS-shaped unit (W = 128, 25 M elements): 2880 columns leave a
    64-column strip at the end of every row of tiles, so full and masked items alternate."""
    u = Unit.from_workload(WORKLOADS[4])
    try:
        run_steps(u, 0, 1400, hypers(2, lr=3e-4), "gpt-oss rank 0")
    finally:
        u.close()


def test_adam8_deepseek_shared_expert_rows():
    """Config 5 (W = 1024): the ranks that hold the shared expert's matrices, whose granularity is
    one row and whose state blocks are therefore runs of 128 along each row, next to the last
    routed expert's 32x32 tiles."""
    wl = WORKLOADS[5]
    u = Unit.from_workload(wl)
    try:
        first_shared = len(wl.tensors) - 3
        l = u.oracle.offsets[first_shared]
        ranks = sorted({l // u.S - 1, l // u.S, (u.oracle.offsets[-1] + u.specs[-1].e - 1) // u.S})
        for k in ranks:
            run_steps(u, int(k), 1500 + int(k), hypers(2, lr=3e-4), f"deepseek rank {k}")
    finally:
        u.close()


@pytest.mark.parametrize("case", range(len(UNITS)))
def test_state_codec_units_every_rank(case):
    """rs_state_quantize / rs_state_dequantize against the oracle's codec, both maps, bit for bit."""
    tensors, world, A = UNITS[case]
    u = Unit(tensors, world, 16, 1, A)
    try:
        S = u.S
        for k in range(world):
            pay = np.zeros(S, dtype=bool)
            for _, _, d, n in u.oracle.rank_segments(k):
                pay[d:d + n] = True
            lo, hi = OA.state_range(u.oracle, k)
            rng = np.random.default_rng(7000 + 10 * case + k)
            for unsigned in (False, True):
                x = (rng.standard_normal(S) * 1e-3).astype(np.float32)
                if unsigned:
                    x = x * x
                x[pay & (rng.random(S) < 0.02)] = 0.0
                x[~pay] = np.nan
                pad_codes = np.full(S, 0x55, np.uint8 if unsigned else np.int8)
                say(f"state codec unit{case} rank {k} unsigned={unsigned}")
                d_codes = torch.from_numpy(pad_codes.copy()).cuda()
                d_am = torch.full((hi - lo + 1,), 7.0, dtype=torch.float32, device="cuda")
                B.rs_state_quantize(u.plan, k, torch.from_numpy(x).cuda(), unsigned, d_codes, d_am)
                torch.cuda.synchronize()
                want_c, want_a = OA.quantise_shard(u.oracle, k, x, pad_codes, not unsigned)
                diff(d_codes.cpu().numpy(), want_c, "codes")
                diff(d_am.cpu().numpy()[:hi - lo].view(np.uint32), want_a.view(np.uint32), "absmax")
                assert d_am.cpu().numpy()[hi - lo] == 7.0
                d_out = torch.full((S,), 9.0, dtype=torch.float32, device="cuda")
                B.rs_state_dequantize(u.plan, k, d_codes, d_am, unsigned, d_out)
                torch.cuda.synchronize()
                want = OA.dequantise_shard(u.oracle, k, want_c, want_a, np.full(S, 9.0, np.float32), not unsigned)
                diff(d_out.cpu().numpy().view(np.uint32), want.view(np.uint32), "dequantised")
    finally:
        u.close()


def test_state_codec_feeds_the_adam_step():
    """Moments quantised by rs_state_quantize are the state rs_adam8_step continues from."""
    u = Unit(UNITS[0][0], UNITS[0][1])
    try:
        S, k = u.S, 2
        lo, hi = OA.state_range(u.oracle, k)
        rng = np.random.default_rng(8123)
        m0 = (rng.standard_normal(S) * 1e-3).astype(np.float32)
        v0 = ((rng.standard_normal(S) * 1e-3) ** 2).astype(np.float32)
        g = (rng.standard_normal(S) * 1e-3).astype(np.float32)
        w = (rng.standard_normal(S) * 0.02).astype(np.float32)
        mc, vc = torch.zeros(S, dtype=torch.int8, device="cuda"), torch.zeros(S, dtype=torch.uint8, device="cuda")
        am, av = (torch.zeros(hi - lo, dtype=torch.float32, device="cuda") for _ in range(2))
        B.rs_state_quantize(u.plan, k, torch.from_numpy(m0).cuda(), False, mc, am)
        B.rs_state_quantize(u.plan, k, torch.from_numpy(v0).cuda(), True, vc, av)
        d_w = torch.from_numpy(w).cuda()
        d_p = torch.zeros(S, dtype=torch.bfloat16, device="cuda")
        h = OA.Hyper(lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.0, step=5)
        B.rs_adam8_step(u.plan, k, (h.lr, h.beta1, h.beta2, h.eps, h.weight_decay, h.step),
                        torch.from_numpy(g).cuda(), d_w, d_p, mc, vc, am, av)
        torch.cuda.synchronize()
        omc, oam = OA.quantise_shard(u.oracle, k, m0, np.zeros(S, np.int8), True)
        ovc, oav = OA.quantise_shard(u.oracle, k, v0, np.zeros(S, np.uint8), False)
        ow, opb, omc, ovc, oam, oav = OA.adam8_step_shard(u.oracle, k, g, w, np.zeros(S, np.uint16), omc, ovc, oam, oav, h)
        diff(d_w.cpu().numpy().view(np.uint32), ow.view(np.uint32), "master")
        diff(mc.cpu().numpy(), omc, "m codes")
        diff(vc.cpu().numpy(), ovc, "v codes")
        diff(am.cpu().numpy().view(np.uint32), oam.view(np.uint32), "m absmax")
    finally:
        u.close()


@pytest.mark.parametrize("seed", range(12))
def test_adam8_random_units(seed):
    """Random units of tensors that carry 8-bit state in every granularity, two steps on a few ranks."""
    import random
    rnd = random.Random(6000 + seed)
    n = rnd.randint(1, 6)
    tensors = []
    for _ in range(n):
        kind = rnd.random()
        if kind < 0.25:
            tensors.append((rnd.randint(1, 3000), 0, rnd.choice([MODE_1x128, MODE_32x32])))
        elif kind < 0.65:
            tensors.append((rnd.randint(1, 300), rnd.choice([8, 24, 30, 32, 40, 100, 128, 130, 256, 300, 1100]),
                            rnd.choice([MODE_32x32, MODE_32x32, MODE_128x128])))
        else:
            tensors.append((rnd.randint(1, 90), rnd.choice([8, 40, 128, 200, 333]), MODE_1x128))
    world = rnd.choice([1, 2, 3, 4, 7, 16])
    A = rnd.choice([0, 0, 0, 1])
    u = Unit(tensors, world, 16, 1, A)
    try:
        say(f"random unit {seed}: {tensors} W={world} A={A} S={u.S}")
        assert B.rs_plan_state_bases(u.plan) == OA.state_bases(u.oracle)
        for k in sorted(set(rnd.sample(range(world), min(world, 2)) + [0, world - 1])):
            run_steps(u, k, 500 * seed + k, hypers(2), f"random{seed}")
    finally:
        u.close()
