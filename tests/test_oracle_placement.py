"""Pins of the placement oracle (Section 4: composing with Shard(dim > 0); Algorithm 2's
SelectRoot; the RaggedShard(r) buffer) against brute force, closed forms and textbook bounds."""
import itertools
import random

import numpy as np
import pytest

from oracle import placement as pl
from oracle import plan as op


# ---- Shard(dim > 0): granularity that never cuts into the dimension ---------------------------

@pytest.mark.parametrize("shape,dim", [((6, 4), 1), ((5, 3, 4), 1), ((5, 3, 4), 2), ((2, 3, 2, 5), 2)])
@pytest.mark.parametrize("g_user", [1, 2, 3, 4, 6, 8, 16])
def test_granularity_is_the_smallest_multiple_whose_boundaries_stay_outside_the_dimension(shape, dim, g_user):
    g = pl.shard_dim_granularity(shape, dim, g_user)
    # the same tensor made long along dimension 0, so that every candidate step has many
    # boundaries inside it
    tall = (2 * g_user * int(np.prod(shape[1:])),) + tuple(shape[1:])
    e = int(np.prod(tall))

    def never_cuts(step):
        # every boundary j*step inside the tensor has zero coordinates along dimensions >= dim
        coords = np.unravel_index(np.arange(step, e, step), tall)
        return not any(c.any() for c in coords[dim:])

    assert never_cuts(g)
    assert [c for c in range(g_user, g, g_user) if never_cuts(c)] == []


def test_granularity_closed_forms():
    # 2-D, Shard(1): whole local rows; rows of 128-tiles when the user asks for 128 rows' worth
    assert pl.shard_dim_granularity((4096, 512), 1, 1) == 512
    assert pl.shard_dim_granularity((4096, 512), 1, 128 * 512) == 128 * 512
    assert pl.shard_dim_granularity((4096, 96), 1, 128) == 384
    # expert-major 3-D tensor sharded along the hidden dimension: whole (hidden, ffn) planes
    assert pl.shard_dim_granularity((8, 64, 48), 1, 1) == 64 * 48
    assert pl.shard_dim_granularity((8, 64, 48), 2, 32) == 96
    with pytest.raises(ValueError):
        pl.shard_dim_granularity((8, 8), 0, 1)
    with pytest.raises(ValueError):
        pl.shard_dim_granularity((8, 8), 2, 1)


def test_plan_with_that_granularity_keeps_rows_whole():
    # a (R, C/tp) local shard planned with the helper's granularity: every rank boundary inside
    # the tensor falls between rows
    R, C = 100, 72
    g = pl.shard_dim_granularity((R, C), 1, 16)
    specs = [op.TensorSpec(R, C, op.BLOCK_EXPLICIT, g), op.TensorSpec(300, 0, op.BLOCK_1x128)]
    p = op.make_plan(specs, 7, 16, 2)
    l = p.offsets[0]
    for k in range(1, 7):
        b = k * p.S
        if l < b < l + R * C:
            assert (b - l) % C == 0


# ---- SelectRoot: longest-processing-time-first ---------------------------------------------

def brute_force_makespan(costs, world):
    best = None
    for assign in itertools.product(range(world), repeat=len(costs)):
        loads = [0] * world
        for c, k in zip(costs, assign):
            loads[k] += c
        best = max(loads) if best is None else min(best, max(loads))
    return best


def test_cost_counts_the_three_products_of_one_iteration():
    # X is a x b with a <= b: X X^T is a*a*b multiply-adds, (X X^T)^2 a*a*a, the update a*a*b
    for r, c in [(3, 5), (5, 3), (4, 4), (1, 9), (128, 512)]:
        a, b = min(r, c), max(r, c)
        assert pl.newton_schulz_cost(r, c) == a * a * b + a ** 3 + a * a * b
    assert pl.newton_schulz_cost(7, 11) == pl.newton_schulz_cost(11, 7)


@pytest.mark.parametrize("seed", range(30))
def test_roots_within_grahams_bound_of_the_optimum(seed):
    rng = random.Random(seed)
    world = rng.randint(1, 3)
    n = rng.randint(1, 7)
    shapes = [(rng.randint(1, 40), rng.choice([0, rng.randint(1, 40)])) for _ in range(n)]
    roots, loads = pl.select_roots(shapes, world)
    mats = [t for t in range(n) if shapes[t][1] > 0]
    assert all(roots[t] == -1 for t in range(n) if shapes[t][1] == 0)
    assert all(0 <= roots[t] < world for t in mats)
    costs = [pl.newton_schulz_cost(*shapes[t]) for t in mats]
    # loads are the sums of what was assigned
    for k in range(world):
        assert loads[k] == sum(c for t, c in zip(mats, costs) if roots[t] == k)
    if mats:
        opt = brute_force_makespan(costs, world)
        # list scheduling in descending order: makespan <= (4/3 - 1/(3 m)) * optimum
        assert 3 * world * max(loads) <= (4 * world - 1) * opt


def test_roots_special_cases():
    same = [(8, 8)] * 10
    roots, loads = pl.select_roots(same, 4)
    assert roots == [0, 1, 2, 3, 0, 1, 2, 3, 0, 1]                        # equal costs: round robin
    assert max(loads) - min(loads) == pl.newton_schulz_cost(8, 8)
    roots, _ = pl.select_roots([(4, 4), (9, 9), (6, 6)], 8)               # more devices than tensors
    assert sorted(roots) == [0, 1, 2] and roots[1] == 0                    # the largest goes first
    roots, loads = pl.select_roots([(5, 0), (7, 0)], 3)
    assert roots == [-1, -1] and loads == [0, 0, 0]
    roots, loads = pl.select_roots([(3, 4), (5, 6)], 1)
    assert roots == [0, 0]


# ---- RaggedShard(r): every tensor whole on its root ---------------------------------------------

@pytest.mark.parametrize("seed", range(20))
def test_rooted_plan_is_a_valid_layout_with_every_tensor_on_its_root(seed):
    rng = random.Random(100 + seed)
    m = rng.randint(1, 6)
    n = rng.randint(1, 9)
    specs = []
    for _ in range(n):
        if rng.random() < 0.25:
            specs.append(op.TensorSpec(rng.randint(1, 700), 0, op.BLOCK_1x128))
        else:
            specs.append(op.TensorSpec(rng.randint(1, 70), rng.randint(1, 90),
                                       rng.choice([op.BLOCK_WHOLE, op.BLOCK_128x128, op.BLOCK_32x32])))
    roots = [rng.randrange(m) for _ in range(n)]
    A = rng.choice([1, 4, 8])
    p = pl.rooted_plan(specs, m, roots, 16, 2, A)
    tensors = [(s.e, s.g) for s in specs]
    assert op.layout_violations(tensors, p.offsets, m, p.S, p.g_coll, A) == []
    for t, s in enumerate(specs):
        assert roots[t] * p.S <= p.offsets[t] and p.offsets[t] + s.e <= (roots[t] + 1) * p.S
    # buffer order is increasing offsets, and within a device the caller's order
    order = p.buffer_order()
    assert [p.offsets[t] for t in order] == sorted(p.offsets)
    for a, b in zip(order, order[1:]):
        assert (roots[a], a) < (roots[b], b)
    # S cannot shrink by a whole unit: some device needs more than S - g_coll elements
    need = [0] * m
    for t in order:
        need[roots[t]] = p.offsets[t] + specs[t].e - roots[t] * p.S
    assert p.S - p.g_coll < max(need) <= p.S
    # every rank's segments are whole tensors
    for k in range(m):
        for t, src_off, dst_off, cnt in p.rank_segments(k):
            assert roots[t] == k and src_off == 0 and cnt == specs[t].e


def test_rooted_plan_closed_forms():
    specs = [op.TensorSpec(10, 10, op.BLOCK_WHOLE), op.TensorSpec(3, 7, op.BLOCK_WHOLE),
             op.TensorSpec(20, 5, op.BLOCK_WHOLE)]
    # all on one device: S = aligned sum
    p = pl.rooted_plan(specs, 4, [2, 2, 2], 16, 2, 8)
    assert p.offsets == [2 * p.S, 2 * p.S + 104, 2 * p.S + 128] and p.S == 232
    # one per device: S = the largest tensor rounded to the unit
    p = pl.rooted_plan(specs, 3, [0, 1, 2], 16, 2)
    assert p.S == 104 and p.offsets == [0, 104, 208]
    with pytest.raises(ValueError):
        pl.rooted_plan(specs, 3, [0, 1, 3])
