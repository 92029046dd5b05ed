"""GPU parity at the full sizes of the benchmark configurations, in the launch configuration
bench.py times (same plans, same entry points, whole-unit launches).

Config 2 is checked element by element on a whole unit against the numpy oracle.  Configs 3-5 are
checked element by element too, on EVERY tensor of the unit and on the whole region of the rank:
the unit stays on the device (inputs drawn there with torch's seeded generator), tensors are
streamed to the host one at a time and compared with the plain-C oracle (oracle/c, which
tests/test_oracle_c.py holds bit for bit against the numpy oracle); a few tensors and one stretch
of each reduce also go through the numpy oracle itself.  Every test builds what it needs, so any
of them can run alone."""
import numpy as np
import pytest
import torch

from oracle import c_oracle as OC
from oracle import dbuffer as OD
from oracle import fp8 as OF
from oracle import plan as OP
from paper_2602_22437_amd import binding as B
from workloads import WORKLOADS, gen_params, gen_partial

from fused_check import order_free_fused_check
from gpu_util import Unit, bits_of, say, to_dev_bf16

pytestmark = pytest.mark.gpu
REDUCE_TOL = 1e-5


# ---------------------------------------------------------------------------------------------
# config 2: Llama-3-8B-shaped unit, W = 64 - full element-by-element parity on unit 0
# ---------------------------------------------------------------------------------------------

class Cfg2:
    """Unit 0 of configuration 2 on both sides; every stage is built on first use and kept."""

    def __init__(self):
        self.wl = WORKLOADS[2]
        say("config 2: generating unit 0 on the host")
        self.unit = Unit.from_workload(self.wl)
        self.params = gen_params(self.wl, seed=1)
        self._packed = self._quantised = None

    def packed(self):
        """(device DBuffer, oracle DBuffer bits)"""
        if self._packed is None:
            u = self.unit
            say("config 2: pack")
            dev = [to_dev_bf16(p) for p in self.params]
            dbuf = torch.full((u.total,), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
            B.rs_pack(u.plan, u.table(dev), dbuf)
            torch.cuda.synchronize()
            self._packed = (dbuf, OD.ragged_pack(self.params, u.oracle.offsets, u.total))
        return self._packed

    def quantised(self):
        """(device codes, device scales, oracle codes, oracle scales) of the whole unit"""
        if self._quantised is None:
            u = self.unit
            dbuf, db_bits = self.packed()
            nb = B.rs_plan_num_scales(u.plan)
            codes = torch.full((u.total,), 0xAB, dtype=torch.uint8, device="cuda")
            scales = torch.full((nb,), float("nan"), dtype=torch.float32, device="cuda")
            say("config 2: quantize all ranks")
            B.rs_quantize(u.plan, -1, dbuf, codes, scales)
            torch.cuda.synchronize()
            say("config 2: oracle quantisation of the whole unit")
            wc, ws = OF.block_quant_all(u.oracle, db_bits)
            self._quantised = (codes, scales, wc, ws)
        return self._quantised

    def close(self):
        self.unit.close()
        self._packed = self._quantised = self.params = None


@pytest.fixture(scope="module")
def cfg2():
    state = Cfg2()
    yield state
    state.close()
    torch.cuda.empty_cache()


def test_config2_pack_and_unpack_bf16(cfg2):
    u = cfg2.unit
    dbuf, want = cfg2.packed()
    assert np.array_equal(bits_of(dbuf), want)
    say("config 2: unpack_bf16")
    outs = [torch.empty(p.size, dtype=torch.bfloat16, device="cuda") for p in cfg2.params]
    B.rs_unpack_bf16(u.plan, dbuf, u.table(outs))
    torch.cuda.synchronize()
    for o, p in zip(outs, cfg2.params):
        assert np.array_equal(bits_of(o), p)


@pytest.mark.parametrize("rank", [0, 40, 63])       # rank 63 holds padding only
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
    # and against the definition alone, whatever the summation order
    n = order_free_fused_check(u.oracle, u.specs, rank, lambda a, b: np.ascontiguousarray(parts[:, a:b]),
                               codes.cpu().numpy(), scales.cpu().numpy()[:hi - lo], f"config 2 rank {rank}", reducer=OC)
    say(f"config 2: fused reduce + quantise, order-free check on {n} elements")
    assert n == int(pay.sum())


def test_config2_quantize_all_and_by_rank(cfg2):
    u = cfg2.unit
    dbuf, _ = cfg2.packed()
    codes, scales, wc, ws = cfg2.quantised()
    assert np.array_equal(scales.cpu().numpy().view(np.uint32), ws.view(np.uint32))
    assert np.array_equal(codes.cpu().numpy(), wc)
    for k in (0, 4, 63):                     # the launch bench.py times is the rank-0 one
        say(f"config 2: quantize rank {k}")
        lo, hi = B.rs_plan_scale_range(u.plan, k)
        c = torch.full((u.S,), 0xCD, dtype=torch.uint8, device="cuda")
        s = torch.full((max(1, hi - lo),), float("nan"), dtype=torch.float32, device="cuda")
        B.rs_quantize(u.plan, k, dbuf[k * u.S:(k + 1) * u.S], c, s)
        torch.cuda.synchronize()
        assert np.array_equal(c.cpu().numpy(), wc[k * u.S:(k + 1) * u.S])
        assert np.array_equal(s.cpu().numpy()[:hi - lo].view(np.uint32), ws[lo:hi].view(np.uint32))


def test_config2_dequant_unpack(cfg2):
    u = cfg2.unit
    codes, scales, want_codes, want_scales = cfg2.quantised()
    outs = [torch.empty(p.size, dtype=torch.bfloat16, device="cuda") for p in cfg2.params]
    say("config 2: dequant_unpack")
    B.rs_unpack(u.plan, codes, scales, u.table(outs))
    torch.cuda.synchronize()
    for i, (spec, l, sb) in enumerate(zip(u.specs, u.oracle.offsets, u.oracle.scale_bases())):
        say(f"config 2: oracle dequantise tensor {i}")
        want = OF.dequantise_tensor(want_codes[l:l + spec.e], want_scales[sb:sb + spec.num_blocks], spec)
        assert np.array_equal(bits_of(outs[i]), want), f"tensor {i}"
    say("config 2: unpack_f32")
    outs32 = [torch.empty(p.size, dtype=torch.float32, device="cuda") for p in cfg2.params]
    B.rs_unpack_f32(u.plan, codes, scales, u.table(outs32))
    torch.cuda.synchronize()
    for i, (spec, l, sb) in enumerate(zip(u.specs, u.oracle.offsets, u.oracle.scale_bases())):
        want = OF.dequantise_tensor_f32(want_codes[l:l + spec.e], want_scales[sb:sb + spec.num_blocks], spec)
        assert np.array_equal(outs32[i].cpu().numpy().view(np.uint32), want.view(np.uint32)), f"fp32 tensor {i}"


def test_config2_batched_launches_as_the_bench_launches_them(cfg2):
    """The launch shapes bench.py times on config 2 besides the per-unit ones: rank 0's shard of
    32 units in ONE block_quant launch, the same for the 8-bit Adam step, and rank 0's region of
    32 units in ONE reduce launch and in ONE fused reduce + quantise launch; every unit's outputs
    against the oracle (quantise, reduce) or against the per-unit launch (fused, Adam)."""
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
    del shards, codes, scales

    # one reduce launch over the region of 32 units; 4 units through the oracle, all against rs_reduce
    W = wl.world
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5)
    parts = [torch.empty(W * S, dtype=torch.bfloat16, device="cuda").normal_(0, 1e-3, generator=gen) for _ in range(n_units)]
    outs = [torch.full((S,), float("nan"), dtype=torch.float32, device="cuda") for _ in range(n_units)]
    rb = B.rs_partials_batch_create(u.plan, rank, parts, S, outs)
    say("config 2: reduce_batch")
    B.rs_reduce_batch(u.plan, rb)
    torch.cuda.synchronize()
    B.rs_partials_batch_destroy(rb)
    single = torch.empty(S, dtype=torch.float32, device="cuda")
    segs = u.oracle.rank_segments(rank)
    for unit in range(n_units):
        B.rs_reduce(u.plan, rank, parts[unit], S, single)
        torch.cuda.synchronize()
        assert torch.equal(single.view(torch.int32), outs[unit].view(torch.int32)), f"unit {unit}: batch != rs_reduce"
        if unit % 8 == 0:
            sub = bits_of(parts[unit]).reshape(W, S)
            got = outs[unit].cpu().numpy()
            err = np.abs(got.astype(np.float64) - OC.shard_reduce(sub, segs))
            assert np.all(err <= REDUCE_TOL * OC.shard_reduce_abs_sum(sub)), f"unit {unit}"
            assert np.array_equal(got.view(np.uint32), OC.shard_reduce_f32_ordered(sub, segs).view(np.uint32))
    # the fused reduce + quantise over the same 32 regions in one launch: every unit equal to
    # its own rs_reduce_quantize (which the test above holds against the oracle at this size),
    # means equal to the reduce's
    say("config 2: reduce_quantize_batch")
    f_codes = [torch.full((S,), 0xEE, dtype=torch.uint8, device="cuda") for _ in range(n_units)]
    f_scales = [torch.full((hi - lo,), float("nan"), dtype=torch.float32, device="cuda") for _ in range(n_units)]
    f_means = [torch.full((S,), float("nan"), dtype=torch.float32, device="cuda") for _ in range(n_units)]
    pin = B.rs_partials_batch_create(u.plan, rank, parts, S, f_means)
    pout = B.rs_shard_batch_create(u.plan, rank, f_means, f_codes, f_scales)   # shard pointers are not read
    B.rs_reduce_quantize_batch(u.plan, pin, pout, True)
    torch.cuda.synchronize()
    B.rs_partials_batch_destroy(pin)
    B.rs_shard_batch_destroy(pout)
    one_c = torch.empty(S, dtype=torch.uint8, device="cuda")
    one_s = torch.empty(hi - lo, dtype=torch.float32, device="cuda")
    for unit in range(n_units):
        B.rs_reduce_quantize(u.plan, rank, parts[unit], S, one_c, one_s)
        torch.cuda.synchronize()
        assert torch.equal(f_codes[unit], one_c), f"unit {unit}: fused batch codes"
        assert torch.equal(f_scales[unit].view(torch.int32), one_s.view(torch.int32)), f"unit {unit}: fused batch scales"
        assert torch.equal(f_means[unit].view(torch.int32), outs[unit].view(torch.int32)), f"unit {unit}: fused batch mean"
    del parts, outs, f_codes, f_scales, f_means

    slo, shi = B.rs_plan_state_range(u.plan, rank)
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
# helpers for the configurations that stay on the device
# ---------------------------------------------------------------------------------------------

def device_params(wl, seed):
    gen = torch.Generator(device="cuda")
    gen.manual_seed(seed)
    return [torch.empty(t.numel, dtype=torch.bfloat16, device="cuda").normal_(0, wl.sigma, generator=gen)
            for t in wl.tensors]


def gaps_are_zero(u, buf):
    """Every padding interval of the buffer (between tensors and after the last) is all zero."""
    flat = buf.view(torch.int16) if buf.dtype == torch.bfloat16 else buf
    cur = 0
    for l, t in sorted(zip(u.oracle.offsets, range(len(u.specs)))):
        if l > cur:
            assert int(torch.count_nonzero(flat[cur:l])) == 0, f"padding before offset {l}"
        cur = l + u.specs[t].e
    if cur < u.total:
        assert int(torch.count_nonzero(flat[cur:])) == 0, "padding at the end of the buffer"


def block_shape(spec):
    """(rows, cols, block height, block width) of a tensor as the C oracle's matrix quantiser sees it"""
    if spec.cols == 0:
        return 1, spec.rows, 1, 128
    return (spec.rows, spec.cols, 128, 128) if spec.mode == OP.BLOCK_128x128 else (spec.rows, spec.cols, 1, 128)


def check_reduce_whole_region(u, wl, rank, partials, out, chunk, numpy_too=True):
    """The whole region of the rank, streamed to the host in column chunks: zero on padding, within
    the tolerance of the float64 mean, bit-equal to the stated fp32 order (C oracle; the first
    chunk that holds payload also through the numpy oracle).  Returns the elements compared."""
    segs = u.oracle.rank_segments(rank)
    W, S = wl.world, u.S
    pv = partials.view(W, S)
    done = 0
    for a in range(0, S, chunk):
        b = min(S, a + chunk)
        local = []
        for t, so, do, n in segs:
            x, y = max(do, a), min(do + n, b)
            if x < y:
                local.append((t, 0, x - a, y - x))
        got = out[a:b].cpu().numpy()
        if not local:
            assert not got.any(), f"padding {a}:{b}"
            done += b - a
            continue
        sub = bits_of(pv[:, a:b].contiguous().view(-1)).reshape(W, b - a)
        pay = np.zeros(b - a, dtype=bool)
        for _, _, d, n in local:
            pay[d:d + n] = True
        assert np.all(got[~pay] == 0), f"padding inside {a}:{b}"
        want = OC.shard_reduce(sub, local)
        err = np.abs(got.astype(np.float64) - want.astype(np.float64))
        # the C mean is the float64 mean rounded to fp32: half an ulp of slack on top of the bound
        bound = REDUCE_TOL * OC.shard_reduce_abs_sum(sub) + np.abs(want).astype(np.float64) * 2.0 ** -24
        assert np.all(err <= bound), f"chunk {a}:{b}"
        ordered = OC.shard_reduce_f32_ordered(sub, local)
        assert np.array_equal(got.view(np.uint32), ordered.view(np.uint32)), f"chunk {a}:{b} order"
        if numpy_too:
            w = min(b - a, 1 << 16)
            clip = [(t, 0, d, min(n, w - d)) for t, _, d, n in local if d < w]
            if clip:
                sw = np.ascontiguousarray(sub[:, :w])
                assert np.all(np.abs(got[:w].astype(np.float64) - OD.shard_reduce(sw, clip)) <=
                              REDUCE_TOL * OD.shard_reduce_abs_sum(sw)), "numpy oracle"
                assert np.array_equal(got[:w].view(np.uint32), OD.shard_reduce_f32_ordered(sw, clip).view(np.uint32))
                numpy_too = False
        done += b - a
    return done


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
        for t, (spec, l) in enumerate(zip(u.specs, u.oracle.offsets)):   # every tensor, on the host
            want = OD.ragged_pack([bits_of(src[t])], [0], spec.e)
            assert np.array_equal(bits_of(dbuf[l:l + spec.e]), want), f"tensor {t}"
        gaps_are_zero(u, dbuf)
        say("config 3: unpack_bf16")
        outs = [torch.full_like(s, 1.0) for s in src]
        B.rs_unpack_bf16(u.plan, dbuf, u.table(outs))
        torch.cuda.synchronize()
        for t, (o, s) in enumerate(zip(outs, src)):
            assert np.array_equal(bits_of(o), bits_of(s)), f"tensor {t}"
        del outs, dbuf
        # every matrix sits whole on one rank
        for t, (spec, l) in enumerate(zip(u.specs, u.oracle.offsets)):
            if spec.cols:
                assert l // u.S == (l + spec.e - 1) // u.S
        for rank in (0, 3, 31):                      # rank 31 holds nothing: all zeros, no reads
            say(f"config 3: reduce rank {rank}, whole region")
            gen = torch.Generator(device="cuda")
            gen.manual_seed(100 + rank)
            partials = torch.empty(wl.world * u.S, dtype=torch.bfloat16, device="cuda").normal_(0, 1e-3, generator=gen)
            out = torch.full((u.S,), float("nan"), dtype=torch.float32, device="cuda")
            B.rs_reduce(u.plan, rank, partials, u.S, out)
            torch.cuda.synchronize()
            if not u.oracle.rank_segments(rank):
                assert int(torch.count_nonzero(out)) == 0
            else:
                n = check_reduce_whole_region(u, wl, rank, partials, out, 1 << 22)
                assert n == u.S
            del partials, out
        with pytest.raises(B.RaggedShardError) as e:
            B.rs_quantize(u.plan, 0, src[0], src[0], src[0])
        assert e.value.code == B.RS_EUNSUPPORTED
    finally:
        u.close()
        torch.cuda.empty_cache()


# ---------------------------------------------------------------------------------------------
# configs 4 and 5: MoE units, all four ops, every tensor element by element
# ---------------------------------------------------------------------------------------------

class MoE:
    """One MoE unit on the device after pack, quantise (all ranks) and dequant_unpack."""
    live = None

    def __init__(self, idx):
        if MoE.live is not None:          # one large unit at a time on the card
            MoE.live.close()
        MoE.live = self
        self.idx = idx
        self.wl = wl = WORKLOADS[idx]
        self.u = u = Unit.from_workload(wl)
        say(f"config {idx}: {len(u.specs)} tensors, W={wl.world}, S={u.S}, total={u.total}")
        self.src = device_params(wl, 10 + idx)
        self.dbuf = torch.full((u.total,), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
        B.rs_pack(u.plan, u.table(self.src), self.dbuf)
        nb = B.rs_plan_num_scales(u.plan)
        self.codes = torch.full((u.total,), 0xAB, dtype=torch.uint8, device="cuda")
        self.scales = torch.full((nb,), float("nan"), dtype=torch.float32, device="cuda")
        say(f"config {idx}: quantize all ranks, nb={nb}")
        B.rs_quantize(u.plan, -1, self.dbuf, self.codes, self.scales)
        self.dst = [torch.empty_like(s) for s in self.src]
        say(f"config {idx}: dequant_unpack")
        B.rs_unpack(u.plan, self.codes, self.scales, u.table(self.dst))
        torch.cuda.synchronize()
        self.sb = u.oracle.scale_bases()

    def close(self):
        if self.u is not None:
            self.u.close()
        self.u = self.src = self.dbuf = self.codes = self.scales = self.dst = None
        if MoE.live is self:
            MoE.live = None
        torch.cuda.empty_cache()


_moe_cache = {}


def moe(idx):
    st = _moe_cache.get(idx)
    if st is None or st.u is None:
        st = _moe_cache[idx] = MoE(idx)
    return st


@pytest.fixture(scope="module", autouse=True)
def _release_moe_units():
    yield
    for st in _moe_cache.values():
        st.close()
    _moe_cache.clear()


def check_tensor(st, t, numpy_too=False):
    """Pack, codes, scales and dequantised values of tensor t against the oracle, every element."""
    u = st.u
    spec, l = u.specs[t], u.oracle.offsets[t]
    src = bits_of(st.src[t])
    assert np.array_equal(bits_of(st.dbuf[l:l + spec.e]), OC.ragged_pack([src], [0], spec.e)), f"pack of tensor {t}"
    R, C, bh, bw = block_shape(spec)
    wc, ws = OC.quantise_matrix(src.reshape(R, C), bh, bw)
    assert np.array_equal(st.codes[l:l + spec.e].cpu().numpy(), wc.reshape(-1)), f"codes of tensor {t}"
    got_s = st.scales[st.sb[t]:st.sb[t + 1]].cpu().numpy()
    assert np.array_equal(got_s.view(np.uint32), ws.reshape(-1).view(np.uint32)), f"scales of tensor {t}"
    want = OC.dequantise_matrix(wc, ws, bh, bw)
    assert np.array_equal(bits_of(st.dst[t]), want.reshape(-1)), f"unpack of tensor {t}"
    if numpy_too:       # the numpy oracle itself on this tensor
        nc, ns = OF.quantise_tensor(src, spec)
        assert np.array_equal(nc, wc.reshape(-1)) and np.array_equal(ns.view(np.uint32), ws.reshape(-1).view(np.uint32))
        assert np.array_equal(OF.dequantise_tensor(nc, ns, spec), want.reshape(-1))
    return spec.e


MOE_CHUNKS = {4: 4, 5: 8}


@pytest.mark.parametrize("idx,chunk", [(i, c) for i in (4, 5) for c in range(MOE_CHUNKS[i])])
def test_moe_unit_every_tensor(idx, chunk):
    """Tensors chunk, chunk + k, chunk + 2k, ... of the unit (k chunks cover all of them)."""
    st = moe(idx)
    u, wl = st.u, st.wl
    n = len(u.specs)
    mine = list(range(chunk, n, MOE_CHUNKS[idx]))
    # through the numpy oracle as well: the first tensor of the chunk, and in configuration 5 the
    # shared expert's row-block matrices (the only 1x128 blocks on matrices in the configurations)
    also = {mine[0]} | ({768, 769, 770} & set(mine) if idx == 5 else set())
    done = 0
    for i, t in enumerate(mine):
        done += check_tensor(st, t, numpy_too=t in also)
        if i % 32 == 0:
            say(f"config {idx} chunk {chunk}: tensor {t} done ({i + 1} of {len(mine)})")
    say(f"config {idx} chunk {chunk}: {len(mine)} tensors, {done} elements = "
        f"{100.0 * done / u.oracle.payload:.1f} % of the unit compared element by element "
        f"(all chunks together: 100 %)")


@pytest.mark.parametrize("idx", [4, 5])
def test_moe_unit_padding_and_rank_launch(idx):
    st = moe(idx)
    u, wl = st.u, st.wl
    gaps_are_zero(u, st.dbuf)
    gaps_are_zero(u, st.codes)
    assert not bool(torch.isnan(st.scales).any())
    k = wl.rank
    lo, hi = B.rs_plan_scale_range(u.plan, k)
    say(f"config {idx}: quantize rank {k} alone")
    c_r = torch.full((u.S,), 0xCD, dtype=torch.uint8, device="cuda")
    s_r = torch.full((max(1, hi - lo),), float("nan"), dtype=torch.float32, device="cuda")
    B.rs_quantize(u.plan, k, st.dbuf[k * u.S:(k + 1) * u.S], c_r, s_r)
    torch.cuda.synchronize()
    assert torch.equal(c_r, st.codes[k * u.S:(k + 1) * u.S])
    assert torch.equal(s_r[:hi - lo].view(torch.int32), st.scales[lo:hi].view(torch.int32))
    # the launch bench.py times in the step: rank k's shard of all the layers it holds, one launch.
    # Shard 0 is the unit's own (already held against the oracle through st.codes), the others are
    # fresh draws with +0 on the region's padding; every shard must equal its own rs_quantize.
    import bench
    n_sh = bench.QUANT_SHARDS[idx]
    say(f"config {idx}: quantize_batch over rank {k}'s shard of {n_sh} units")
    pay = torch.zeros(u.S, dtype=torch.bool, device="cuda")
    for _, _, d, n in u.oracle.rank_segments(k):
        pay[d:d + n] = True
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4242 + idx)
    shards = [st.dbuf[k * u.S:(k + 1) * u.S]]
    for _ in range(n_sh - 1):
        x = torch.empty(u.S, dtype=torch.bfloat16, device="cuda").normal_(0, wl.sigma, generator=gen)
        shards.append(torch.where(pay, x, torch.zeros_like(x)))
    codes = [torch.full((u.S,), 0xEE, dtype=torch.uint8, device="cuda") for _ in range(n_sh)]
    scales = [torch.full((max(1, hi - lo),), float("nan"), dtype=torch.float32, device="cuda") for _ in range(n_sh)]
    batch = B.rs_shard_batch_create(u.plan, k, shards, codes, scales)
    B.rs_quantize_batch(u.plan, batch)
    torch.cuda.synchronize()
    B.rs_shard_batch_destroy(batch)
    assert torch.equal(codes[0], c_r) and torch.equal(scales[0].view(torch.int32), s_r.view(torch.int32))
    for i in range(1, n_sh):
        B.rs_quantize(u.plan, k, shards[i], c_r, s_r)
        torch.cuda.synchronize()
        assert torch.equal(codes[i], c_r), f"shard {i}: batch != rs_quantize"
        assert torch.equal(scales[i].view(torch.int32), s_r.view(torch.int32)), f"shard {i} scales"
    # one of the fresh shards through the oracle as well (whole shard)
    oc, os_ = OF.block_quant_shard(u.oracle, k, bits_of(shards[n_sh - 1]))
    assert np.array_equal(codes[n_sh - 1].cpu().numpy(), oc)
    assert np.array_equal(scales[n_sh - 1].cpu().numpy()[:hi - lo].view(np.uint32), os_.view(np.uint32))
    del shards, codes, scales
    # the tensors that touch a rank boundary among the first 8 ranks, the rank of interest, and the
    # ends of the unit lie in the chunks above; name them so a reader can see they are covered
    touching = sorted({t for kk in range(1, 9) for t, (s, l) in enumerate(zip(u.specs, u.oracle.offsets))
                       if l <= kk * u.S <= l + s.e} | {t for t, _, _, _ in u.oracle.rank_segments(k)} | {0, len(u.specs) - 1})
    say(f"config {idx}: boundary / rank-of-interest tensors {touching} are among the tensors compared")


@pytest.mark.parametrize("idx", [4, 5])
def test_moe_unit_reduce_whole_region(idx):
    st = moe(idx)
    u, wl = st.u, st.wl
    k = wl.rank
    lo, hi = B.rs_plan_scale_range(u.plan, k)
    say(f"config {idx}: reduce rank {k} with {wl.world} partials, whole region")
    gen = torch.Generator(device="cuda")
    gen.manual_seed(77)
    partials = torch.empty(wl.world * u.S, dtype=torch.bfloat16, device="cuda").normal_(0, 1e-3, generator=gen)
    out = torch.full((u.S,), float("nan"), dtype=torch.float32, device="cuda")
    B.rs_reduce(u.plan, k, partials, u.S, out)
    torch.cuda.synchronize()
    assert not bool(torch.isnan(out).any())
    chunk = max(2048, (1 << 28) // wl.world // 2048 * 2048)        # 512 MB of partials per chunk
    n = check_reduce_whole_region(u, wl, k, partials, out, chunk)
    say(f"config {idx}: reduce compared on {n} of {u.S} elements of the region")
    assert n == u.S

    say(f"config {idx}: fused reduce + quantise of rank {k}")
    c_f = torch.full((u.S,), 0xEE, dtype=torch.uint8, device="cuda")
    s_f = torch.full((max(1, hi - lo),), float("nan"), dtype=torch.float32, device="cuda")
    mean = torch.full((u.S,), float("nan"), dtype=torch.float32, device="cuda")
    B.rs_reduce_quantize(u.plan, k, partials, u.S, c_f, s_f, mean)
    torch.cuda.synchronize()
    assert torch.equal(mean.view(torch.int32), out.view(torch.int32)), "fused mean != rs_reduce"
    assert not bool(torch.isnan(s_f[:hi - lo]).any())
    # every tiled segment of the region against the oracle's quantisation of the ordered mean
    # (numpy, fp32 input), a row of tiles at a time on the first and last rows of tiles, and the
    # whole region against the definition alone (order-free)
    rows_2d = partials.view(wl.world, u.S)
    sb = u.oracle.scale_bases()
    for t, src_off, dst_off, n_seg in u.oracle.rank_segments(k):
        spec = u.specs[t]
        if spec.mode != OP.BLOCK_128x128:
            continue
        C, g = spec.cols, 128 * spec.cols
        n_rows_of_tiles = -(-n_seg // g)
        for br in sorted({0, n_rows_of_tiles - 1}):
            a, b = dst_off + br * g, min(dst_off + (br + 1) * g, dst_off + n_seg)
            win = rows_2d[:, a:b].contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
            want_mean = OD.shard_reduce_f32_ordered(win, [(0, 0, 0, b - a)])
            wc, ws = OF.quantise_matrix_f32(want_mean.reshape(-1, C), 128, 128)
            assert np.array_equal(c_f[a:b].cpu().numpy(), wc.reshape(-1)), f"fused codes, tensor {t}"
            s0 = sb[t] + (src_off // g + br) * spec.nbc - lo
            assert np.array_equal(s_f[s0:s0 + spec.nbc].cpu().numpy().view(np.uint32),
                                  ws.reshape(-1).view(np.uint32)), f"fused scales, tensor {t}"
    codes_h, scales_h = c_f.cpu().numpy(), s_f.cpu().numpy()[:hi - lo]

    def get_parts(a, b):
        return bits_of(rows_2d[:, a:b].contiguous().view(-1)).reshape(wl.world, b - a)
    checked = order_free_fused_check(u.oracle, u.specs, k, get_parts, codes_h, scales_h, f"config {idx} rank {k}",
                                     reducer=OC)
    assert checked == sum(seg[3] for seg in u.oracle.rank_segments(k))
    say(f"config {idx}: fused reduce + quantise, order-free check on {checked} elements (the rank's whole payload)")
