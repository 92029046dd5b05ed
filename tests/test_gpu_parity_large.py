"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (same plans, same entry points, whole-unit launches).

Config 2 (the benched workload) is checked element by element on a whole unit.  Configs 3-5
are too large for a full CPU pass within a test's time limit, so whole-buffer properties are
checked on the device (payload preserved, padding zero) and sampled tensors / windows are
compared element by element with the oracle.  Inputs for configs 3-5 are drawn on the device
with torch's seeded generator and copied to the host for the oracle."""
import numpy as np
import pytest
import torch

from oracle import dbuffer as OD
from oracle import fp8 as OF
from oracle import plan as OP
from paper_2602_22437_amd import binding as B
from workloads import WORKLOADS, gen_params, gen_partial

from gpu_util import Unit, bits_of, say, to_dev_bf16

pytestmark = pytest.mark.gpu
REDUCE_TOL = 1e-5


# ---------------------------------------------------------------------------------------------
# config 2: Llama-3-8B-shaped unit, W = 64 - full element-by-element parity on unit 0
# ---------------------------------------------------------------------------------------------

class Cfg2:
    unit = None
    params = None
    db_bits = None
    dbuf = None
    codes = None
    scales = None


@pytest.fixture(scope="module")
def cfg2():
    wl = WORKLOADS[2]
    say("config 2: generating unit 0 on the host")
    Cfg2.unit = Unit.from_workload(wl)
    Cfg2.params = gen_params(wl, seed=1)
    yield Cfg2
    Cfg2.unit.close()
    Cfg2.params = Cfg2.db_bits = Cfg2.dbuf = Cfg2.codes = Cfg2.scales = None


def test_config2_pack_and_unpack_bf16(cfg2):
    u = cfg2.unit
    say("config 2: pack")
    dev = [to_dev_bf16(p) for p in cfg2.params]
    dbuf = torch.full((u.total,), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
    B.rs_pack(u.plan, u.table(dev), dbuf)
    torch.cuda.synchronize()
    want = OD.ragged_pack(cfg2.params, u.oracle.offsets, u.total)
    assert np.array_equal(bits_of(dbuf), want)
    cfg2.db_bits, cfg2.dbuf = want, dbuf
    say("config 2: unpack_bf16")
    outs = [torch.empty(p.size, dtype=torch.bfloat16, device="cuda") for p in cfg2.params]
    B.rs_unpack_bf16(u.plan, dbuf, u.table(outs))
    torch.cuda.synchronize()
    for o, p in zip(outs, cfg2.params):
        assert np.array_equal(bits_of(o), p)


@pytest.mark.parametrize("rank", [0, 63])
def test_config2_reduce(cfg2, rank):
    wl, u = WORKLOADS[2], cfg2.unit
    say(f"config 2: reduce rank {rank}, generating {wl.world} partials")
    parts = np.stack([gen_partial(wl, 1, w, u.S, unit=rank) for w in range(wl.world)])
    out = torch.full((u.S,), float("nan"), dtype=torch.float32, device="cuda")
    B.rs_reduce(u.plan, rank, to_dev_bf16(parts.reshape(-1)), u.S, out)
    torch.cuda.synchronize()
    segs = u.oracle.rank_segments(rank)
    want = OD.shard_reduce(parts, segs)
    got = out.cpu().numpy()
    pay = np.zeros(u.S, dtype=bool)
    for _, _, d, n in segs:
        pay[d:d + n] = True
    assert np.all(got[~pay] == 0)
    err = np.abs(got.astype(np.float64) - want)
    assert np.all(err <= REDUCE_TOL * OD.shard_reduce_abs_sum(parts))
    ordered = OD.shard_reduce_f32_ordered(parts, segs)
    assert np.array_equal(got.view(np.uint32), ordered.view(np.uint32)), "fp32 summation order differs"
    say(f"config 2: fused reduce + quantise rank {rank}")
    lo, hi = u.oracle.scale_range(rank)
    codes = torch.full((u.S,), 0xEE, dtype=torch.uint8, device="cuda")
    scales = torch.full((max(hi - lo, 1),), float("nan"), dtype=torch.float32, device="cuda")
    B.rs_reduce_quantize(u.plan, rank, to_dev_bf16(parts.reshape(-1)), u.S, codes, scales)
    torch.cuda.synchronize()
    want_c, want_s = OF.block_quant_shard(u.oracle, rank, ordered, f32=True)
    assert np.array_equal(scales.cpu().numpy()[:hi - lo].view(np.uint32), want_s.view(np.uint32))
    assert np.array_equal(codes.cpu().numpy(), want_c)


def test_config2_quantize_all_and_by_rank(cfg2):
    u = cfg2.unit
    assert cfg2.dbuf is not None, "pack test must run first"
    nb = B.rs_plan_num_scales(u.plan)
    codes = torch.full((u.total,), 0xAB, dtype=torch.uint8, device="cuda")
    scales = torch.full((nb,), float("nan"), dtype=torch.float32, device="cuda")
    say("config 2: quantize all ranks")
    B.rs_quantize(u.plan, -1, cfg2.dbuf, codes, scales)
    torch.cuda.synchronize()
    say("config 2: oracle quantisation of the whole unit")
    wc, ws = OF.block_quant_all(u.oracle, cfg2.db_bits)
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), ws.view(np.uint32))
    assert np.array_equal(codes.cpu().numpy(), wc)
    cfg2.codes, cfg2.scales = codes, scales
    cfg2.want_codes, cfg2.want_scales = wc, ws
    for k in (0, 4, 63):                     # the launch bench.py times is the rank-0 one
        say(f"config 2: quantize rank {k}")
        lo, hi = B.rs_plan_scale_range(u.plan, k)
        c = torch.full((u.S,), 0xCD, dtype=torch.uint8, device="cuda")
        s = torch.full((max(1, hi - lo),), float("nan"), dtype=torch.float32, device="cuda")
        B.rs_quantize(u.plan, k, cfg2.dbuf[k * u.S:(k + 1) * u.S], c, s)
        torch.cuda.synchronize()
        assert np.array_equal(c.cpu().numpy(), wc[k * u.S:(k + 1) * u.S])
        assert np.array_equal(s.cpu().numpy()[:hi - lo].view(np.uint32), ws[lo:hi].view(np.uint32))


def test_config2_dequant_unpack(cfg2):
    u = cfg2.unit
    assert cfg2.codes is not None, "quantize test must run first"
    outs = [torch.empty(p.size, dtype=torch.bfloat16, device="cuda") for p in cfg2.params]
    say("config 2: dequant_unpack")
    B.rs_unpack(u.plan, cfg2.codes, cfg2.scales, u.table(outs))
    torch.cuda.synchronize()
    for i, (spec, l, sb) in enumerate(zip(u.specs, u.oracle.offsets, u.oracle.scale_bases())):
        say(f"config 2: oracle dequantise tensor {i}")
        want = OF.dequantise_tensor(cfg2.want_codes[l:l + spec.e],
                                    cfg2.want_scales[sb:sb + spec.num_blocks], spec)
        assert np.array_equal(bits_of(outs[i]), want), f"tensor {i}"
    say("config 2: unpack_f32")
    outs32 = [torch.empty(p.size, dtype=torch.float32, device="cuda") for p in cfg2.params]
    B.rs_unpack_f32(u.plan, cfg2.codes, cfg2.scales, u.table(outs32))
    torch.cuda.synchronize()
    for i, (spec, l, sb) in enumerate(zip(u.specs, u.oracle.offsets, u.oracle.scale_bases())):
        want = OF.dequantise_tensor_f32(cfg2.want_codes[l:l + spec.e],
                                        cfg2.want_scales[sb:sb + spec.num_blocks], spec)
        assert np.array_equal(outs32[i].cpu().numpy().view(np.uint32), want.view(np.uint32)), f"fp32 tensor {i}"


# ---------------------------------------------------------------------------------------------
# helpers for the sampled configurations
# ---------------------------------------------------------------------------------------------

def device_params(wl, seed):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    return [torch.empty(t.numel, dtype=torch.bfloat16, device="cuda").normal_(0, wl.sigma, generator=gen)
            for t in wl.tensors]


def sample_tensors(u, wl, cap):
    """The tensors compared one by one: those overlapping the rank of interest, the first and
    the last, those touching a shard boundary among the first 8 ranks, then every 16th."""
    n = len(u.specs)
    pick = []

    def add(t):
        if t not in pick and len(pick) < cap:
            pick.append(t)
    for t, _, _, _ in u.oracle.rank_segments(wl.rank):
        add(t)
    add(0)
    add(n - 1)
    for k in range(1, 9):
        b = k * u.S
        for t, (s, l) in enumerate(zip(u.specs, u.oracle.offsets)):
            if l <= b <= l + s.e:
                add(t)
    for t in range(0, n, 16):
        add(t)
    return pick


def check_pack_window(u, dbuf, src, t):
    """DBuffer around tensor t (with the padding on both sides) against the oracle pack."""
    spec, l = u.specs[t], u.oracle.offsets[t]
    prev_end = 0 if t == 0 else u.oracle.offsets[t - 1] + u.specs[t - 1].e
    next_start = u.total if t == len(u.specs) - 1 else u.oracle.offsets[t + 1]
    a = max(prev_end, l - 4096)
    b = min(next_start, l + spec.e + 4096)
    want = OD.ragged_pack([bits_of(src[t])], [l - a], b - a)
    assert np.array_equal(bits_of(dbuf[a:b]), want), f"pack window of tensor {t}"


def padding_is_zero_and_payload_kept(u, dbuf, src):
    """Whole-buffer property on the device: as many non-zeros in the DBuffer as in the sources
    (so nothing but zeros in the padding, given the sampled tensors match)."""
    nz_buf = 0
    v = dbuf.view(torch.int16)
    step = 1 << 28
    for a in range(0, v.numel(), step):
        nz_buf += int(torch.count_nonzero(v[a:a + step]))
    nz_src = sum(int(torch.count_nonzero(s.view(torch.int16))) for s in src)
    assert nz_buf == nz_src


def gaps_are_zero(u, buf):
    """Every padding interval of the buffer (between tensors and after the last) is all zero."""
    flat = buf.view(torch.int16) if buf.dtype == torch.bfloat16 else buf
    cur = 0
    for spec, l in zip(u.specs, u.oracle.offsets):
        if l > cur:
            assert int(torch.count_nonzero(flat[cur:l])) == 0, f"padding before offset {l}"
        cur = l + spec.e
    if cur < u.total:
        assert int(torch.count_nonzero(flat[cur:])) == 0, "padding at the end of the buffer"


def check_reduce_windows(u, wl, rank, partials, out, windows):
    segs = u.oracle.rank_segments(rank)
    W, S = wl.world, u.S
    pv = partials.view(W, S)
    for a, b in windows:
        sub = bits_of(pv[:, a:b].contiguous().view(-1)).reshape(W, b - a)
        local = []
        for t, so, do, n in segs:
            x, y = max(do, a), min(do + n, b)
            if x < y:
                local.append((t, 0, x - a, y - x))
        want = OD.shard_reduce(sub, local)
        got = out[a:b].cpu().numpy()
        pay = np.zeros(b - a, dtype=bool)
        for _, _, d, n in local:
            pay[d:d + n] = True
        assert np.all(got[~pay] == 0)
        err = np.abs(got.astype(np.float64) - want)
        assert np.all(err <= REDUCE_TOL * OD.shard_reduce_abs_sum(sub)), f"window {a}:{b}"
        ordered = OD.shard_reduce_f32_ordered(sub, local)
        assert np.array_equal(got.view(np.uint32), ordered.view(np.uint32)), f"window {a}:{b} order"


def reduce_windows(u, rank, count, width):
    """Windows over the rank's region: its start, its end, every segment edge, evenly spread."""
    S = u.S
    pts = {0, max(0, S - width)}
    for _, _, d, n in u.oracle.rank_segments(rank):
        for p in (d, d + n):
            pts.add(min(max(0, p - width // 2) // 8 * 8, max(0, S - width)))
    for i in range(count):
        pts.add((S - width) * i // max(1, count - 1) // 8 * 8)
    return [(p, min(S, p + width)) for p in sorted(pts)]


def test_config2_batched_quantize_and_adam_as_the_bench_launches_them(cfg2):
    """The launch shapes bench.py times on config 2 besides the per-unit ones: rank 0's shard of
    32 units in ONE block_quant launch, and the same for the 8-bit Adam step; every unit's
    outputs against the oracle (quantise) or against the per-unit launch (Adam)."""
    from workloads import normal_bf16
    u, wl = cfg2.unit, WORKLOADS[2]
    rank, n_units, S = wl.rank, wl.units, cfg2.unit.S
    lo, hi = u.oracle.scale_range(rank)
    say(f"config 2: {n_units} rank-{rank} shards on the host")
    host = [normal_bf16(77, 2, 0, unit, S, 0.02) for unit in range(n_units)]
    pay = np.zeros(S, dtype=bool)
    for _, _, d, n in u.oracle.rank_segments(rank):
        pay[d:d + n] = True
    for h in host:
        h[~pay] = 0                           # a packed buffer holds +0 on padding
    shards = [to_dev_bf16(h) for h in host]
    codes = [torch.full((S,), 0xEE, dtype=torch.uint8, device="cuda") for _ in range(n_units)]
    scales = [torch.full((hi - lo,), float("nan"), dtype=torch.float32, device="cuda") for _ in range(n_units)]
    batch = B.rs_shard_batch_create(u.plan, rank, shards, codes, scales)
    say("config 2: quantize_batch")
    B.rs_quantize_batch(u.plan, batch)
    torch.cuda.synchronize()
    B.rs_shard_batch_destroy(batch)
    for unit in range(n_units):
        oc, os_ = OF.block_quant_shard(u.oracle, rank, host[unit])
        assert np.array_equal(codes[unit].cpu().numpy(), oc), f"unit {unit} codes"
        assert np.array_equal(scales[unit].cpu().numpy().view(np.uint32), os_.view(np.uint32)), f"unit {unit} scales"

    slo, shi = B.rs_plan_state_range(u.plan, rank)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(99)

    def state():
        return dict(
            g=[torch.empty(S, dtype=torch.float32, device="cuda").normal_(0, 1e-3, generator=gen) for _ in range(n_units)],
            w=[torch.empty(S, dtype=torch.float32, device="cuda").normal_(0, 0.02, generator=gen) for _ in range(n_units)],
            p=[torch.zeros(S, dtype=torch.bfloat16, device="cuda") for _ in range(n_units)],
            mc=[torch.zeros(S, dtype=torch.int8, device="cuda") for _ in range(n_units)],
            vc=[torch.zeros(S, dtype=torch.uint8, device="cuda") for _ in range(n_units)],
            am=[torch.zeros(shi - slo, dtype=torch.float32, device="cuda") for _ in range(n_units)],
            av=[torch.zeros(shi - slo, dtype=torch.float32, device="cuda") for _ in range(n_units)])
    a = state()
    b = {k: [t.clone() for t in v] for k, v in a.items()}
    ab = B.rs_adam8_batch_create(u.plan, rank, a["g"], a["w"], a["p"], a["mc"], a["vc"], a["am"], a["av"])
    for step in (1, 2):
        hyper = (3e-4, 0.9, 0.95, 1e-8, 0.1, step)
        say(f"config 2: adam8_step_batch, step {step}")
        B.rs_adam8_step_batch(u.plan, ab, hyper)
        for i in range(n_units):
            B.rs_adam8_step(u.plan, rank, hyper, b["g"][i], b["w"][i], b["p"][i], b["mc"][i], b["vc"][i],
                            b["am"][i], b["av"][i])
        torch.cuda.synchronize()
        for k in ("w", "p", "mc", "vc", "am", "av"):
            for i in range(n_units):
                x, y = a[k][i], b[k][i]
                if x.dtype == torch.bfloat16:
                    x, y = x.view(torch.int16), y.view(torch.int16)
                elif x.dtype == torch.float32:
                    x, y = x.view(torch.int32), y.view(torch.int32)
                assert torch.equal(x, y), f"{k} of unit {i} differs at step {step}"
    B.rs_adam8_batch_destroy(ab)


# ---------------------------------------------------------------------------------------------
# config 3: whole-matrix sharding (Muon / Shampoo style), W = 32, bf16 only
# ---------------------------------------------------------------------------------------------

def test_config3_whole_matrix_pack_reduce_unpack():
    wl = WORKLOADS[3]
    u = Unit.from_workload(wl)
    try:
        src = device_params(wl, 3)
        say(f"config 3: pack, total={u.total}")
        dbuf = torch.full((u.total,), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
        B.rs_pack(u.plan, u.table(src), dbuf)
        torch.cuda.synchronize()
        for t in range(len(u.specs)):
            check_pack_window(u, dbuf, src, t)
        padding_is_zero_and_payload_kept(u, dbuf, src)
        say("config 3: unpack_bf16")
        outs = [torch.full_like(s, 1.0) for s in src]
        B.rs_unpack_bf16(u.plan, dbuf, u.table(outs))
        torch.cuda.synchronize()
        for o, s in zip(outs, src):
            assert torch.equal(o.view(torch.int16), s.view(torch.int16))
        del outs, dbuf
        # every matrix sits whole on one rank
        for t, (spec, l) in enumerate(zip(u.specs, u.oracle.offsets)):
            if spec.cols:
                assert l // u.S == (l + spec.e - 1) // u.S
        for rank in (0, 3, 31):                      # rank 31 holds nothing: all zeros, no reads
            say(f"config 3: reduce rank {rank}")
            gen = torch.Generator(device="cuda")
            gen.manual_seed(100 + rank)
            partials = torch.empty(wl.world * u.S, dtype=torch.bfloat16, device="cuda").normal_(0, 1e-3, generator=gen)
            out = torch.full((u.S,), float("nan"), dtype=torch.float32, device="cuda")
            B.rs_reduce(u.plan, rank, partials, u.S, out)
            torch.cuda.synchronize()
            if not u.oracle.rank_segments(rank):
                assert int(torch.count_nonzero(out)) == 0
            else:
                check_reduce_windows(u, wl, rank, partials, out, reduce_windows(u, rank, 24, 16384))
            del partials, out
        with pytest.raises(B.RaggedShardError) as e:
            B.rs_quantize(u.plan, 0, src[0], src[0], src[0])
        assert e.value.code == B.RS_EUNSUPPORTED
    finally:
        u.close()


# ---------------------------------------------------------------------------------------------
# configs 4 and 5: MoE units, all four ops, sampled element-by-element parity
# ---------------------------------------------------------------------------------------------

@pytest.mark.parametrize("idx,cap", [(4, 10), (5, 8)])
def test_moe_units_sampled(idx, cap):
    wl = WORKLOADS[idx]
    u = Unit.from_workload(wl)
    try:
        say(f"config {idx}: {len(u.specs)} tensors, W={wl.world}, S={u.S}, total={u.total}")
        src = device_params(wl, 10 + idx)
        pick = sample_tensors(u, wl, cap)
        share = sum(u.specs[t].e for t in pick) / u.oracle.payload
        say(f"config {idx}: sampled tensors {pick} ({100 * share:.1f} % of the unit's elements)")
        dbuf = torch.full((u.total,), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
        B.rs_pack(u.plan, u.table(src), dbuf)
        torch.cuda.synchronize()
        for t in pick:
            check_pack_window(u, dbuf, src, t)
        padding_is_zero_and_payload_kept(u, dbuf, src)
        gaps_are_zero(u, dbuf)

        nb = B.rs_plan_num_scales(u.plan)
        codes = torch.full((u.total,), 0xAB, dtype=torch.uint8, device="cuda")
        scales = torch.full((nb,), float("nan"), dtype=torch.float32, device="cuda")
        say(f"config {idx}: quantize all ranks, nb={nb}")
        B.rs_quantize(u.plan, -1, dbuf, codes, scales)
        torch.cuda.synchronize()
        assert not bool(torch.isnan(scales).any())
        k = wl.rank
        lo, hi = B.rs_plan_scale_range(u.plan, k)
        say(f"config {idx}: quantize rank {k} alone")
        c_r = torch.full((u.S,), 0xCD, dtype=torch.uint8, device="cuda")
        s_r = torch.full((max(1, hi - lo),), float("nan"), dtype=torch.float32, device="cuda")
        B.rs_quantize(u.plan, k, dbuf[k * u.S:(k + 1) * u.S], c_r, s_r)
        torch.cuda.synchronize()
        assert torch.equal(c_r, codes[k * u.S:(k + 1) * u.S])
        assert torch.equal(s_r[:hi - lo].view(torch.int32), scales[lo:hi].view(torch.int32))

        dst = [torch.empty_like(s) for s in src]
        say(f"config {idx}: dequant_unpack")
        B.rs_unpack(u.plan, codes, scales, u.table(dst))
        torch.cuda.synchronize()
        sb = u.oracle.scale_bases()
        for t in pick:
            spec, l = u.specs[t], u.oracle.offsets[t]
            say(f"config {idx}: oracle quantise/dequantise tensor {t} ({spec.rows}x{spec.cols})")
            wc, ws = OF.quantise_tensor(bits_of(src[t]), spec)
            assert np.array_equal(codes[l:l + spec.e].cpu().numpy(), wc), f"codes of tensor {t}"
            assert np.array_equal(scales[sb[t]:sb[t + 1]].cpu().numpy().view(np.uint32), ws.view(np.uint32))
            assert np.array_equal(bits_of(dst[t]), OF.dequantise_tensor(wc, ws, spec)), f"unpack of tensor {t}"
        gaps_are_zero(u, codes)
        del dst
        say(f"config {idx}: reduce rank {k} with {wl.world} partials")
        gen = torch.Generator(device="cuda")
        gen.manual_seed(77)
        partials = torch.empty(wl.world * u.S, dtype=torch.bfloat16, device="cuda").normal_(0, 1e-3, generator=gen)
        out = torch.full((u.S,), float("nan"), dtype=torch.float32, device="cuda")
        B.rs_reduce(u.plan, k, partials, u.S, out)
        torch.cuda.synchronize()
        assert not bool(torch.isnan(out).any())
        check_reduce_windows(u, wl, k, partials, out, reduce_windows(u, k, 12, 4096))

        say(f"config {idx}: fused reduce + quantise of rank {k}")
        c_f = torch.full((u.S,), 0xEE, dtype=torch.uint8, device="cuda")
        s_f = torch.full((max(1, hi - lo),), float("nan"), dtype=torch.float32, device="cuda")
        mean = torch.full((u.S,), float("nan"), dtype=torch.float32, device="cuda")
        B.rs_reduce_quantize(u.plan, k, partials, u.S, c_f, s_f, mean)
        torch.cuda.synchronize()
        assert torch.equal(mean.view(torch.int32), out.view(torch.int32)), "fused mean != rs_reduce"
        assert not bool(torch.isnan(s_f[:hi - lo]).any())
        # whole rows of tiles against the oracle: the first and the last of every tiled segment
        rows_2d = partials.view(wl.world, u.S)
        sb = u.oracle.scale_bases()
        for t, src_off, dst_off, n in u.oracle.rank_segments(k):
            spec = u.specs[t]
            if spec.mode != OP.BLOCK_128x128:
                continue
            C, g = spec.cols, 128 * spec.cols
            n_rows_of_tiles = -(-n // g)
            for br in sorted({0, n_rows_of_tiles - 1}):
                a, b = dst_off + br * g, min(dst_off + (br + 1) * g, dst_off + n)
                say(f"config {idx}: oracle mean and codes of tensor {t}, row of tiles {src_off // g + br}")
                win = rows_2d[:, a:b].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
                want_mean = OD.shard_reduce_f32_ordered(win, [(0, 0, 0, b - a)])
                wc, ws = OF.quantise_matrix_f32(want_mean.reshape(-1, C), 128, 128)
                assert np.array_equal(c_f[a:b].cpu().numpy(), wc.reshape(-1)), f"fused codes, tensor {t}"
                s0 = sb[t] + (src_off // g + br) * spec.nbc - lo
                assert np.array_equal(s_f[s0:s0 + spec.nbc].cpu().numpy().view(np.uint32),
                                      ws.reshape(-1).view(np.uint32)), f"fused scales, tensor {t}"
    finally:
        u.close()
