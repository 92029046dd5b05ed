"""rs_pack_noalloc (ragged_pack whose tensor -> address table is staged in a fixed array in
device memory instead of one made by hipMalloc) against rs_pack, bit for bit, through the C ABI:
two calls in a row on one GPU, the second on a smaller unit, so that whatever the first call left
in the shared array must not leak into the second."""
import ctypes as C

import numpy as np
import pytest
import torch

from oracle import dbuffer as OD
from paper_2602_22437_amd import binding as B
from workloads import normal_bf16

from gpu_util import Unit, bits_of, say, to_dev_bf16

pytestmark = pytest.mark.gpu


def big_unit_shapes():
    """600 tensors (three staging launches of 256, 256 and 88 pointers): matrices of a few ragged
    shapes in 128x128 mode and 1-D vectors, so the buffer has tensor edges inside granules,
    padding and 16-byte-misaligned tails."""
    shapes = []
    for i in range(600):
        if i % 5 == 4:
            shapes.append((384 + 8 * (i % 7), 0, 0))
        else:
            shapes.append((128 * (1 + i % 3), 128 + 64 * (i % 4), 1))
    return shapes


def run_both(shapes, world, seed, misalign_first=False):
    u = Unit(shapes, world)
    try:
        host = [normal_bf16(seed, 9, 0, t, s.e, 0.02) for t, s in enumerate(u.specs)]
        dev = []
        for t, h in enumerate(host):
            if misalign_first and t == 0:
                # a source that is element- but not 16-byte-aligned takes the per-element path
                raw = torch.zeros(h.size + 8, dtype=torch.bfloat16, device="cuda")
                view = raw[1:1 + h.size]
                view.copy_(to_dev_bf16(h))
                dev.append(view)
            else:
                dev.append(to_dev_bf16(h))
        ref = torch.full((u.total,), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
        got = torch.full((u.total,), -1, dtype=torch.int16, device="cuda").view(torch.bfloat16)
        say(f"rs_pack, {len(shapes)} tensors, W={world}, total={u.total}")
        B.rs_pack(u.plan, u.table(dev), ref)
        say(f"rs_pack_noalloc, {len(shapes)} tensors")
        B.rs_pack_noalloc(u.plan, dev, got)
        torch.cuda.synchronize()
        assert torch.equal(ref.view(torch.int16), got.view(torch.int16))
        # and both equal the definition
        want = OD.ragged_pack(host, u.oracle.offsets, u.total)
        assert np.array_equal(bits_of(got), want)
    finally:
        u.close()


def test_noalloc_pack_equals_pack_on_two_calls_in_a_row():
    run_both(big_unit_shapes(), 8, seed=31, misalign_first=True)
    # the second call is smaller: 6 tensors (the toy unit's shapes), one staging launch
    toy = [(256, 384, 1), (384, 0, 0), (512, 256, 1), (1000, 128, 1), (128, 128, 1), (257, 130, 1)]
    run_both(toy, 4, seed=32)
    # and a larger one again on the same GPU's array
    run_both(big_unit_shapes()[:300], 16, seed=33)


def test_noalloc_pack_argument_checks():
    toy = [(256, 384, 1), (384, 0, 0)]
    u = Unit(toy, 2)
    try:
        src = [torch.zeros(s.e, dtype=torch.bfloat16, device="cuda") for s in u.specs]
        dbuf = torch.zeros(u.total, dtype=torch.bfloat16, device="cuda")
        arr = (C.c_void_p * 2)(src[0].data_ptr(), 0)
        assert B.raw_call("rs_pack_noalloc", u.plan, arr, C.c_void_p(dbuf.data_ptr()), None) == B.RS_EINVAL
        arr = (C.c_void_p * 2)(src[0].data_ptr(), src[1].data_ptr() + 1)
        assert B.raw_call("rs_pack_noalloc", u.plan, arr, C.c_void_p(dbuf.data_ptr()), None) == B.RS_EALIGN
        arr = (C.c_void_p * 2)(src[0].data_ptr(), src[1].data_ptr())
        assert B.raw_call("rs_pack_noalloc", u.plan, arr, C.c_void_p(dbuf.data_ptr() + 2), None) == B.RS_EALIGN
        assert B.raw_call("rs_pack_noalloc", u.plan, None, C.c_void_p(dbuf.data_ptr()), None) == B.RS_EINVAL
        assert B.raw_call("rs_pack_noalloc", None, arr, C.c_void_p(dbuf.data_ptr()), None) == B.RS_EINVAL
    finally:
        u.close()
    # more tensors than the fixed array holds: refused with its own code, nothing launched
    many = [(128, 0, 0)] * (B.RS_NOALLOC_MAX_TENSORS + 1)
    u = Unit(many, 2)
    try:
        one = torch.zeros(128, dtype=torch.bfloat16, device="cuda")
        dbuf = torch.zeros(u.total, dtype=torch.bfloat16, device="cuda")
        with pytest.raises(B.RaggedShardError) as e:
            B.rs_pack_noalloc(u.plan, [one] * len(many), dbuf)
        assert e.value.code == B.RS_ETOOBIG
        assert "rs_pack_noalloc" in B.rs_strerror(B.RS_ETOOBIG)
    finally:
        u.close()
