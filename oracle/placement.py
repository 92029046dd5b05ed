"""Oracle for the placement helpers around the layout plan.  TEST INFRASTRUCTURE ONLY - never
imported by the product.

Three small host-side pieces, each written out from its definition:

  * shard_dim_granularity: composing RaggedShard with an even Shard(dim > 0) (Section 4, the
    paragraph on composing with existing sharding formats, its second case): the granularity is the
    least common multiple of a stride of the tensor and the user's granularity so that a ragged
    boundary never falls inside dimension `dim`.
  * select_roots: SelectRoot of Algorithm 2 (distributed Muon, Section 6.3), of which the paper
    says only that it balances load.
  * rooted_plan: the DBuffer of a group of tensors placed RaggedShard(r_t): all blocks of tensor
    t on device r_t (Section 4: arbitrary sharding distribution; Algorithm 2's redistribute target).

Readings taken where the paper is silent:
  * Keeping dimension dim whole is read as: every ragged boundary, counted in elements of the
    row-major local tensor, has all coordinates along dimensions >= dim equal to zero.  Those
    offsets are the multiples of prod(shape[dim:]) (the stride of dimension dim - 1), so
    g = lcm(prod(shape[dim:]), g_user).
  * Load balancing is longest-processing-time-first list scheduling: 2-D tensors in descending
    cost (equal costs in index order), each to the device with the least accumulated cost (the
    lowest such device).  The cost of an R x C matrix is that of one quintic Newton-Schulz
    iteration on it, in units of two flops: with a = min(R, C), b = max(R, C), the Gram matrix
    costs a*a*b, its square a*a*a and the update a*a*b, together a*a*(2b + a).  1-D tensors are
    not Muon parameters and get root -1.
  * In the rooted DBuffer, device k's region holds the tensors rooted at k in index order, each
    start a multiple of the tensor alignment A; S is the largest region's extent rounded up to
    g_coll.
"""
from __future__ import annotations

from math import gcd, prod
from typing import List, Optional, Sequence, Tuple

from .plan import Plan, TensorSpec


def shard_dim_granularity(shape: Sequence[int], dim: int, g_user: int) -> int:
    if not 0 < dim < len(shape) or g_user <= 0 or any(d <= 0 for d in shape):
        raise ValueError("need 0 < dim < ndim, positive sizes and a positive granularity")
    plane = prod(shape[dim:])
    return plane // gcd(plane, g_user) * g_user


def newton_schulz_cost(rows: int, cols: int) -> int:
    a, b = min(rows, cols), max(rows, cols)
    return a * a * (2 * b + a)


def select_roots(shapes: Sequence[Tuple[int, int]], world: int) -> Tuple[List[int], List[int]]:
    """(root of every tensor, accumulated cost of every device).  shapes: (rows, cols), cols == 0
    marks a 1-D tensor."""
    if world <= 0:
        raise ValueError("world must be positive")
    roots = [-1] * len(shapes)
    loads = [0] * world
    matrices = [t for t, (r, c) in enumerate(shapes) if c > 0]
    matrices.sort(key=lambda t: -newton_schulz_cost(*shapes[t]))          # stable: ties keep index order
    for t in matrices:
        k = min(range(world), key=lambda d: loads[d])                      # min() keeps the lowest of equals
        roots[t] = k
        loads[k] += newton_schulz_cost(*shapes[t])
    return roots, loads


def rooted_plan(specs: Sequence[TensorSpec], m: int, roots: Sequence[int], align_bytes: int = 16,
                min_itemsize: int = 1, tensor_align: Optional[int] = None) -> Plan:
    if align_bytes % min_itemsize != 0:
        raise ValueError("alignment must be a multiple of the item size")
    g_coll = align_bytes // min_itemsize
    A = g_coll if tensor_align is None else tensor_align
    if g_coll % A != 0 or len(roots) != len(specs) or any(not 0 <= r < m for r in roots):
        raise ValueError("bad alignment or roots")
    rel = [0] * len(specs)          # start of every tensor inside its device's region
    extent = [0] * m
    for t, s in enumerate(specs):
        k = roots[t]
        rel[t] = -(-extent[k] // A) * A
        extent[k] = rel[t] + s.e
    S = -(-max(extent) // g_coll) * g_coll
    offsets = [roots[t] * S + rel[t] for t in range(len(specs))]
    perm = sorted(range(len(specs)), key=lambda t: (roots[t], t))
    return Plan(list(specs), m, g_coll, A, S, offsets, perm)
