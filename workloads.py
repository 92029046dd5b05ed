"""Synthetic workloads: the five FSDP-unit configurations and the seeded input generators.

This module holds shapes and random draws only - none of the method's arithmetic - so
that the CPU oracle and the HIP path can be fed the very same inputs without sharing
any code.  Every array is a pure function of (seed, config, role, index): a
counter-based Philox stream keyed by those four integers, so either side can regenerate
any tensor without holding the whole unit.

Shapes stand in for the public model architectures the paper evaluates (Section 6:
LLaMA-3, GPT-OSS-120B, DeepSeek-V3); values are N(0, sigma) rounded to bf16, gradient
partials N(0, 1e-3).  No real weights or datasets are used.

Block modes (same integers as the C ABI): 0 = 1x128, 1 = 128x128, 2 = whole tensor,
3 = explicit granularity, 4 = 32x32 (8-bit optimiser state).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, Tuple

import numpy as np
import torch

MODE_1x128, MODE_128x128, MODE_WHOLE, MODE_EXPLICIT, MODE_32x32 = 0, 1, 2, 3, 4

ROLE_PARAM, ROLE_PARTIAL, ROLE_MISC = 0, 1, 2


@dataclass(frozen=True)
class TensorShape:
    name: str
    rows: int
    cols: int      # 0 => 1-D tensor of `rows` elements
    mode: int

    @property
    def numel(self) -> int:
        return self.rows * self.cols if self.cols else self.rows


@dataclass(frozen=True)
class Workload:
    index: int             # 1-based, as the configurations are numbered
    name: str
    world: int             # W, the FSDP size (m in the paper)
    align_bytes: int
    min_itemsize: int      # narrowest dtype that shares the plan (1 when an FP8 buffer does)
    sigma: float
    rank: int              # the rank whose shard reduce / quantise work on
    quantised: bool
    units: int             # how many such units run back to back
    tensors: Tuple[TensorShape, ...]

    @property
    def numel(self) -> int:
        return sum(t.numel for t in self.tensors)


def _llama_layer(mode2d: int) -> Tuple[TensorShape, ...]:
    h, kv, ffn = 4096, 1024, 14336
    return (
        TensorShape("attn_norm", h, 0, MODE_1x128),
        TensorShape("wq", h, h, mode2d),
        TensorShape("wk", kv, h, mode2d),
        TensorShape("wv", kv, h, mode2d),
        TensorShape("wo", h, h, mode2d),
        TensorShape("ffn_norm", h, 0, MODE_1x128),
        TensorShape("w1", ffn, h, mode2d),
        TensorShape("w3", ffn, h, mode2d),
        TensorShape("w2", h, ffn, mode2d),
    )


def _gpt_oss_unit() -> Tuple[TensorShape, ...]:
    h, nq, nkv, hd, ne = 2880, 64, 8, 64, 128
    ts = [
        TensorShape("wq", nq * hd, h, MODE_128x128),
        TensorShape("wk", nkv * hd, h, MODE_128x128),
        TensorShape("wv", nkv * hd, h, MODE_128x128),
        TensorShape("wo", h, nq * hd, MODE_128x128),
        TensorShape("router", ne, h, MODE_128x128),
    ]
    for i in range(ne):
        ts.append(TensorShape(f"expert{i}.gate_up", 2 * h, h, MODE_128x128))
        ts.append(TensorShape(f"expert{i}.down", h, h, MODE_128x128))
    return tuple(ts)


def _deepseek_unit() -> Tuple[TensorShape, ...]:
    h, inter, ne = 7168, 2048, 256
    ts = []
    for i in range(ne):
        ts.append(TensorShape(f"expert{i}.gate", inter, h, MODE_128x128))
        ts.append(TensorShape(f"expert{i}.up", inter, h, MODE_128x128))
        ts.append(TensorShape(f"expert{i}.down", h, inter, MODE_128x128))
    # the shared expert carries the 1x128 row blocks
    ts.append(TensorShape("shared.gate", inter, h, MODE_1x128))
    ts.append(TensorShape("shared.up", inter, h, MODE_1x128))
    ts.append(TensorShape("shared.down", h, inter, MODE_1x128))
    return tuple(ts)


_TOY = (
    TensorShape("p0", 256, 384, MODE_128x128),
    TensorShape("p1", 384, 0, MODE_1x128),
    TensorShape("p2", 512, 256, MODE_128x128),
    TensorShape("p3", 1000, 128, MODE_128x128),
    TensorShape("p4", 128, 128, MODE_128x128),
    TensorShape("p5", 257, 130, MODE_128x128),
)

WORKLOADS = {
    1: Workload(1, "toy_w4", 4, 16, 1, 0.02, 0, True, 1, _TOY),
    2: Workload(2, "llama3_8b_layer_w64", 64, 16, 1, 0.02, 0, True, 32, _llama_layer(MODE_128x128)),
    3: Workload(3, "llama3_8b_layer_whole_matrix_w32", 32, 16, 2, 0.02, 0, False, 1,
                _llama_layer(MODE_WHOLE)),
    4: Workload(4, "gpt_oss_120b_moe_w128", 128, 16, 1, 0.02, 0, True, 1, _gpt_oss_unit()),
    5: Workload(5, "deepseek_v3_moe_w1024", 1024, 16, 1, 0.006, 511, True, 1, _deepseek_unit()),
}


def _rng(seed: int, config: int, role: int, index: int) -> np.random.Generator:
    ss = np.random.SeedSequence(entropy=[int(seed), int(config), int(role), int(index)])
    return np.random.Generator(np.random.Philox(seed=ss))


def _to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 bit patterns (uint16) with the library's own rounding."""
    t = torch.from_numpy(x).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16)


def normal_bf16(seed: int, config: int, role: int, index: int, n: int, sigma: float) -> np.ndarray:
    """n draws of N(0, sigma) rounded to bf16, returned as uint16 bit patterns."""
    out = np.empty(n, dtype=np.uint16)
    rng = _rng(seed, config, role, index)
    step = 1 << 24
    for a in range(0, n, step):
        b = min(n, a + step)
        x = rng.standard_normal(b - a, dtype=np.float32)
        x *= np.float32(sigma)
        out[a:b] = _to_bf16_bits(x)
    return out


def gen_param(wl: Workload, seed: int, t: int, unit: int = 0) -> np.ndarray:
    """bf16 bits of parameter tensor t (flat, row-major) of unit `unit`."""
    return normal_bf16(seed, wl.index, ROLE_PARAM, unit * 100003 + t, wl.tensors[t].numel, wl.sigma)


def gen_params(wl: Workload, seed: int, unit: int = 0) -> List[np.ndarray]:
    return [gen_param(wl, seed, t, unit) for t in range(len(wl.tensors))]


def gen_partial(wl: Workload, seed: int, w: int, n: int, unit: int = 0) -> np.ndarray:
    """bf16 bits of gradient partial w's copy of one shard region (n = S elements)."""
    return normal_bf16(seed, wl.index, ROLE_PARTIAL, unit * 100003 + w, n, 1e-3)


def uniform_bits(seed: int, config: int, index: int, n: int, lo: int, hi: int) -> np.ndarray:
    """n integers in [lo, hi) - raw material for edge-case tests."""
    return _rng(seed, config, ROLE_MISC, index).integers(lo, hi, size=n, dtype=np.int64)
