"""Helpers for the GPU parity tests: build a unit on both sides (oracle plan + library plan)
and move bit patterns between numpy and device tensors.  No arithmetic of the method here."""
from __future__ import annotations

import sys

import numpy as np
import torch

from oracle import placement as PL
from oracle import plan as P
from paper_2602_22437_amd import binding as B


def say(msg: str) -> None:
    print(f"[gpu-test] {msg}", flush=True)
    sys.stdout.flush()


def to_dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(bits.view(np.int16)).cuda().view(torch.bfloat16)


def bits_of(t: torch.Tensor) -> np.ndarray:
    """uint16 bit patterns of a bf16 device tensor (or uint8 / raw views of others)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    if t.dtype == torch.float32:
        return t.cpu().numpy()
    return t.cpu().numpy()


class Unit:
    """One FSDP unit planned by both sides."""

    def __init__(self, tensors, world, align_bytes=16, min_itemsize=1, tensor_align=0, device=0, order=0,
                 roots=None):
        self.tensors = [tuple(t) for t in tensors]
        self.world = world
        self.specs = [P.TensorSpec(*t) for t in self.tensors]
        if roots is None:
            self.oracle = P.make_plan(self.specs, world, align_bytes, min_itemsize,
                                      tensor_align=tensor_align or None, order=order)
            self.plan = B.rs_plan_create_ordered(self.tensors, world, align_bytes, min_itemsize,
                                                 tensor_align, order)
        else:       # every tensor whole on its root device
            self.oracle = PL.rooted_plan(self.specs, world, roots, align_bytes, min_itemsize,
                                         tensor_align or None)
            self.plan = B.rs_plan_create_rooted(self.tensors, world, roots, align_bytes, min_itemsize,
                                                tensor_align)
        assert B.rs_plan_shard_elems(self.plan) == self.oracle.S
        assert B.rs_plan_offsets(self.plan) == self.oracle.offsets
        B.rs_plan_upload(self.plan, device)
        self.S = self.oracle.S
        self.total = self.oracle.total
        self.tables = []
        self.keep = []

    def table(self, dev_tensors):
        dev_tensors = list(dev_tensors)
        t = B.rs_tensor_table_create(self.plan, dev_tensors)
        self.tables.append(t)
        self.keep.append(dev_tensors)   # the table holds bare addresses: the tensors must outlive it
        return t

    def close(self):
        for t in self.tables:
            B.rs_tensor_table_destroy(t)
        self.tables = []
        self.keep = []
        if self.plan:
            B.rs_plan_destroy(self.plan)
            self.plan = None

    @classmethod
    def from_workload(cls, wl):
        return cls([(t.rows, t.cols, t.mode) for t in wl.tensors], wl.world, wl.align_bytes,
                   wl.min_itemsize)
