"""Every device call writes inside its outputs only: each output buffer is a view into a larger
allocation whose guard bands (64 elements in front and behind, a known pattern) must survive
every operation of the library on a ragged unit, for every rank."""
import numpy as np
import pytest
import torch

from paper_2602_22437_amd import binding as B
from workloads import MODE_128x128, MODE_1x128, normal_bf16

from gpu_util import Unit, say, to_dev_bf16

pytestmark = pytest.mark.gpu
GUARD = 64


class Guarded:
    """A tensor of n elements with guard bands; .t is the 16-byte-aligned payload view."""

    def __init__(self, n, dtype, fill):
        self.n = n
        self.whole = torch.empty(n + 2 * GUARD, dtype=dtype, device="cuda")
        self.pattern = fill
        self.whole.view(torch.uint8).fill_(fill)
        self.t = self.whole[GUARD:GUARD + n]
        assert self.t.data_ptr() % 16 == 0

    def check(self, what):
        raw = self.whole.view(torch.uint8)
        item = self.whole.element_size()
        front, back = raw[:GUARD * item], raw[(GUARD + self.n) * item:]
        assert bool((front == self.pattern).all()) and bool((back == self.pattern).all()), f"guard band hit by {what}"


def test_guard_bands_survive_every_operation():
    tensors = [(257, 136, MODE_128x128), (300, 0, MODE_1x128), (130, 256, MODE_128x128), (40, 200, MODE_1x128)]
    W = 3
    u = Unit(tensors, W)
    try:
        S, total = u.S, u.total
        nb = B.rs_plan_num_scales(u.plan)
        params = [normal_bf16(60, 0, 0, i, s.e, 0.02) for i, s in enumerate(u.specs)]
        src = [to_dev_bf16(p) for p in params]
        tab_src = u.table(src)
        dbuf = Guarded(total, torch.bfloat16, 0x5A)
        codes = Guarded(total, torch.uint8, 0x5A)
        scales = Guarded(nb, torch.float32, 0x5A)
        dst = [Guarded(s.e, torch.bfloat16, 0x5A) for s in u.specs]
        dst32 = [Guarded(s.e, torch.float32, 0x5A) for s in u.specs]
        tab_dst, tab_dst32 = u.table([g.t for g in dst]), u.table([g.t for g in dst32])
        everything = [dbuf, codes, scales] + dst + dst32

        def check_all(what):
            torch.cuda.synchronize()
            for g in everything:
                g.check(what)

        say("group operators")
        B.rs_pack(u.plan, tab_src, dbuf.t); check_all("rs_pack")
        B.rs_pack_scaled(u.plan, tab_src, 0.5, dbuf.t); check_all("rs_pack_scaled")
        B.rs_group_add(u.plan, tab_src, 1.0, dbuf.t); check_all("rs_group_add")
        B.rs_group_scale(u.plan, 2.0, dbuf.t); check_all("rs_group_scale")
        B.rs_group_zero(u.plan, dbuf.t); check_all("rs_group_zero")
        B.rs_pack(u.plan, tab_src, dbuf.t); check_all("rs_pack")
        say("FP8 codec")
        B.rs_quantize(u.plan, -1, dbuf.t, codes.t, scales.t); check_all("rs_quantize all")
        B.rs_unpack(u.plan, codes.t, scales.t, tab_dst); check_all("rs_unpack")
        B.rs_unpack_f32(u.plan, codes.t, scales.t, tab_dst32); check_all("rs_unpack_f32")
        B.rs_unpack_bf16(u.plan, dbuf.t, tab_dst); check_all("rs_unpack_bf16")
        for k in range(W):
            say(f"rank {k}: reduce, shard quantise, optimiser state")
            lo, hi = B.rs_plan_scale_range(u.plan, k)
            slo, shi = B.rs_plan_state_range(u.plan, k)
            parts = torch.randn(W * S, device="cuda").to(torch.bfloat16)
            out = Guarded(S, torch.float32, 0x5A)
            kc, ks = Guarded(S, torch.uint8, 0x5A), Guarded(max(hi - lo, 4), torch.float32, 0x5A)
            master, param = Guarded(S, torch.float32, 0), Guarded(S, torch.bfloat16, 0x5A)
            mc, vc = Guarded(S, torch.int8, 0), Guarded(S, torch.uint8, 0)
            am, av = Guarded(max(shi - slo, 4), torch.float32, 0), Guarded(max(shi - slo, 4), torch.float32, 0)
            mine = [out, kc, ks, master, param, mc, vc, am, av]
            everything.extend(mine)
            B.rs_reduce(u.plan, k, parts, S, out.t); check_all("rs_reduce")
            B.rs_quantize(u.plan, k, dbuf.t[k * S:(k + 1) * S], kc.t, ks.t); check_all("rs_quantize rank")
            B.rs_reduce_quantize(u.plan, k, parts, S, kc.t, ks.t); check_all("rs_reduce_quantize")
            B.rs_reduce_quantize(u.plan, k, parts, S, kc.t, ks.t, out.t); check_all("rs_reduce_quantize + mean")
            B.rs_adam8_step(u.plan, k, (1e-3, 0.9, 0.95, 1e-8, 0.01, 1), out.t, master.t, param.t, mc.t, vc.t,
                            am.t, av.t); check_all("rs_adam8_step")
            B.rs_state_dequantize(u.plan, k, mc.t, am.t, False, out.t); check_all("rs_state_dequantize")
            B.rs_state_quantize(u.plan, k, out.t, False, mc.t, am.t); check_all("rs_state_quantize")
            for g in mine:
                everything.remove(g)
    finally:
        u.close()
