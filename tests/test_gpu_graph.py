"""The device entry points only enqueue kernels (no allocation, no synchronisation, no memset), so a
whole step can be captured into a HIP graph and replayed: every replay must equal the eager calls
on the inputs of that moment, bit for bit."""
import numpy as np
import pytest
import torch

from paper_2602_22437_amd import binding as B
from workloads import MODE_128x128, MODE_1x128, normal_bf16

from gpu_util import Unit, say, to_dev_bf16

pytestmark = pytest.mark.gpu


def fresh_inputs(u, W, rank, seed):
    srcs = [normal_bf16(seed, 1, 0, i, s.e, 0.02) for i, s in enumerate(u.specs)]
    parts = np.stack([normal_bf16(seed, 2, rank, w, u.S, 1e-3) for w in range(W)])
    return srcs, parts


@pytest.mark.parametrize("tensors,W", [
    ([(300, 384, MODE_128x128), (1000, 0, MODE_1x128), (257, 136, MODE_128x128), (64, 256, MODE_1x128)], 4),
    ([(512, 1024, MODE_128x128), (4096, 0, MODE_1x128)], 8),
])
def test_a_captured_step_replays_like_the_eager_calls(tensors, W):
    u = Unit(tensors, W)
    try:
        rank = W - 1
        nb = u.oracle.scale_bases()[-1]
        srcs, parts = fresh_inputs(u, W, rank, 100)
        src_dev = [to_dev_bf16(s) for s in srcs]
        dst_dev = [torch.zeros(s.e, dtype=torch.bfloat16, device="cuda") for s in u.specs]
        tab_src, tab_dst = u.table(src_dev), u.table(dst_dev)
        part_dev = to_dev_bf16(parts.reshape(-1))

        def buffers():
            return dict(dbuf=torch.zeros(u.total, dtype=torch.bfloat16, device="cuda"),
                        dbuf2=torch.zeros(u.total, dtype=torch.bfloat16, device="cuda"),
                        mean=torch.zeros(u.S, dtype=torch.float32, device="cuda"),
                        codes=torch.zeros(u.total, dtype=torch.uint8, device="cuda"),
                        scales=torch.zeros(max(nb, 1), dtype=torch.float32, device="cuda"))
        g_out, e_out = buffers(), buffers()

        def step(o, dst_table):
            B.rs_pack(u.plan, tab_src, o["dbuf"])
            B.rs_pack_noalloc(u.plan, src_dev, o["dbuf2"])
            B.rs_reduce(u.plan, rank, part_dev, u.S, o["mean"])
            B.rs_quantize(u.plan, -1, o["dbuf"], o["codes"], o["scales"])
            B.rs_unpack(u.plan, o["codes"], o["scales"], dst_table)

        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            step(g_out, tab_dst)                       # warm-up outside the capture
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        say("capturing pack, pack_noalloc, reduce, quantize, unpack")
        with torch.cuda.graph(graph):
            step(g_out, tab_dst)
        torch.cuda.synchronize()

        e_dst = [torch.zeros(s.e, dtype=torch.bfloat16, device="cuda") for s in u.specs]
        e_tab = u.table(e_dst)
        for replay in range(4):
            srcs, parts = fresh_inputs(u, W, rank, 200 + replay)     # new values in the same buffers
            for d, s in zip(src_dev, srcs):
                d.copy_(to_dev_bf16(s))
            part_dev.copy_(to_dev_bf16(parts.reshape(-1)))
            for t in list(g_out.values()) + dst_dev:
                t.view(torch.uint8).fill_(0x5A)                       # stale outputs must be overwritten
            torch.cuda.synchronize()
            say(f"replay {replay}")
            graph.replay()
            torch.cuda.synchronize()
            step(e_out, e_tab)                                        # the program's own eager work in between
            torch.cuda.synchronize()
            for k in g_out:
                assert torch.equal(g_out[k].view(torch.uint8), e_out[k].view(torch.uint8)), f"replay {replay}: {k}"
            assert torch.equal(g_out["dbuf"].view(torch.int16), g_out["dbuf2"].view(torch.int16))
            for i, (a, b) in enumerate(zip(dst_dev, e_dst)):
                assert torch.equal(a.view(torch.int16), b.view(torch.int16)), f"replay {replay}: tensor {i}"
    finally:
        u.close()
