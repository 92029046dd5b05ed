"""Host side of the placement helpers (no GPU needed): the library must agree with the oracle on
the Shard(dim > 0) granularity, the roots and the rooted buffer layout, and reject bad input
with error codes."""
import random

import pytest

from oracle import adam8 as OA
from oracle import placement as PL
from oracle import plan as P
from paper_2602_22437_amd import binding as B
from workloads import WORKLOADS


@pytest.mark.parametrize("seed", range(40))
def test_shard_dim_granularity_matches_oracle(seed):
    rnd = random.Random(seed)
    ndim = rnd.randint(2, 4)
    shape = [rnd.randint(1, 96) for _ in range(ndim)]
    dim = rnd.randint(1, ndim - 1)
    g_user = rnd.choice([1, 2, 8, 16, 32, 128, rnd.randint(1, 300)])
    assert B.rs_shard_dim_granularity(shape, dim, g_user) == PL.shard_dim_granularity(shape, dim, g_user)


def test_shard_dim_granularity_errors():
    for shape, dim, g in [([8, 8], 0, 1), ([8, 8], 2, 1), ([8], 0, 1), ([8, 0], 1, 1), ([8, 8], 1, 0)]:
        with pytest.raises(B.RaggedShardError) as ei:
            B.rs_shard_dim_granularity(shape, dim, g)
        assert ei.value.code == B.RS_EINVAL
    with pytest.raises(B.RaggedShardError) as ei:
        B.rs_shard_dim_granularity([2 ** 31, 2 ** 31], 1, 1)
    assert ei.value.code == B.RS_EOVERFLOW
    with pytest.raises(B.RaggedShardError) as ei:
        B.rs_shard_dim_granularity([2 ** 20, 2 ** 20], 1, 2 ** 61 - 1)
    assert ei.value.code == B.RS_EOVERFLOW


@pytest.mark.parametrize("seed", range(40))
def test_select_roots_matches_oracle(seed):
    rnd = random.Random(1000 + seed)
    n = rnd.randint(1, 40)
    world = rnd.choice([1, 2, 3, 8, 64])
    shapes = []
    for _ in range(n):
        r = rnd.choice([1, 7, 64, 64, 128, 4096, rnd.randint(1, 10 ** 5)])
        c = rnd.choice([0, 64, 64, 128, 14336, rnd.randint(1, 10 ** 5)])
        shapes.append((r, c))
    roots, loads = B.rs_select_roots([(r, c, B.RS_BLOCK_WHOLE) for r, c in shapes], world)
    want_roots, want_loads = PL.select_roots(shapes, world)
    assert roots == want_roots
    assert loads == [float(x) for x in want_loads]


def test_select_roots_on_the_paper_shaped_units():
    # the dense layer: seven matrices on 64 devices, each alone; the two vectors are not Muon's
    wl = WORKLOADS[3]
    shapes = [(t.rows, t.cols) for t in wl.tensors]
    roots, loads = B.rs_select_roots([(t.rows, t.cols, B.RS_BLOCK_WHOLE) for t in wl.tensors], wl.world)
    assert roots == PL.select_roots(shapes, wl.world)[0]
    mats = [t for t, (r, c) in enumerate(shapes) if c > 0]
    assert len({roots[t] for t in mats}) == len(mats) and all(roots[t] == -1 for t in range(len(shapes)) if t not in mats)
    # the expert unit: equal experts spread evenly
    wl = WORKLOADS[4]
    shapes = [(t.rows, t.cols) for t in wl.tensors]
    roots, loads = B.rs_select_roots([(t.rows, t.cols, B.RS_BLOCK_WHOLE) for t in wl.tensors], wl.world)
    want_roots, want_loads = PL.select_roots(shapes, wl.world)
    assert roots == want_roots and loads == [float(x) for x in want_loads]
    assert max(loads) <= 4 / 3 * sum(loads) / wl.world + max(PL.newton_schulz_cost(*s) for s in shapes)


def test_select_roots_errors():
    for tensors, world in [([], 4), ([(8, 8, 2)], 0), ([(0, 8, 2)], 2), ([(8, -1, 2)], 2)]:
        with pytest.raises(B.RaggedShardError) as ei:
            B.rs_select_roots(tensors, world)
        assert ei.value.code == B.RS_EINVAL


def has_state(spec):
    try:
        OA.state_runs(spec)
        return True
    except ValueError:
        return False


def random_group(rnd):
    n = rnd.randint(1, 9)
    tensors = []
    for _ in range(n):
        kind = rnd.random()
        if kind < 0.2:
            tensors.append((rnd.randint(1, 700), 0, B.RS_BLOCK_1x128))
        elif kind < 0.5:
            tensors.append((rnd.randint(1, 300), rnd.choice([8, 24, 128, 130, 256]), B.RS_BLOCK_128x128))
        elif kind < 0.7:
            tensors.append((rnd.randint(1, 300), rnd.choice([8, 40, 96, 200]), B.RS_BLOCK_32x32))
        else:
            tensors.append((rnd.randint(1, 80), rnd.randint(1, 80), B.RS_BLOCK_WHOLE))
    return tensors


@pytest.mark.parametrize("seed", range(40))
def test_rooted_plan_matches_oracle(seed):
    rnd = random.Random(2000 + seed)
    tensors = random_group(rnd)
    world = rnd.choice([1, 2, 3, 5, 8, 17])
    roots = [rnd.randrange(world) for _ in tensors]
    align, item = rnd.choice([(16, 1), (16, 2), (32, 2)])
    A = rnd.choice([0, 1, 4, align // item])
    specs = [P.TensorSpec(*t) for t in tensors]
    want = PL.rooted_plan(specs, world, roots, align, item, None if A == 0 else A)
    plan = B.rs_plan_create_rooted(tensors, world, roots, align, item, A)
    try:
        assert B.rs_plan_shard_elems(plan) == want.S
        assert B.rs_plan_offsets(plan) == want.offsets
        assert B.rs_plan_order(plan) == want.buffer_order()
        assert B.rs_plan_payload_elems(plan) == want.payload
        assert B.rs_plan_padding_elems(plan) == want.padding
        assert B.rs_plan_scale_bases(plan) == want.scale_bases()
        for k in range(world):
            assert B.rs_plan_rank_segments(plan, k) == want.rank_segments(k)
            assert B.rs_plan_scale_range(plan, k) == want.scale_range(k)
        if all(has_state(s) for s in specs):
            assert B.rs_plan_state_bases(plan) == OA.state_bases(want)
            for k in range(world):
                assert B.rs_plan_state_range(plan, k) == OA.state_range(want, k)
    finally:
        B.rs_plan_destroy(plan)


def test_roots_then_rooted_plan_on_the_dense_layer():
    # SelectRoot followed by the rooted buffer: S = the largest matrix, one matrix per device
    wl = WORKLOADS[3]
    tensors = [(t.rows, t.cols, B.RS_BLOCK_WHOLE) for t in wl.tensors if t.cols > 0]
    roots, _ = B.rs_select_roots(tensors, wl.world)
    plan = B.rs_plan_create_rooted(tensors, wl.world, roots, wl.align_bytes, wl.min_itemsize)
    try:
        assert B.rs_plan_shard_elems(plan) == max(r * c for r, c, _ in tensors)
        offs = B.rs_plan_offsets(plan)
        S = B.rs_plan_shard_elems(plan)
        assert offs == [roots[t] * S for t in range(len(tensors))]
    finally:
        B.rs_plan_destroy(plan)


def test_rooted_plan_errors():
    t = [(8, 8, B.RS_BLOCK_WHOLE), (4, 4, B.RS_BLOCK_WHOLE)]
    for roots in ([0, 2], [-1, 0]):
        with pytest.raises(B.RaggedShardError) as ei:
            B.rs_plan_create_rooted(t, 2, roots)
        assert ei.value.code == B.RS_EINVAL
    with pytest.raises(B.RaggedShardError) as ei:
        B.rs_plan_create_rooted([(2 ** 30, 2 ** 30, B.RS_BLOCK_WHOLE)] * 2, 8, [0, 0])
    assert ei.value.code == B.RS_EOVERFLOW
