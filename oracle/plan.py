"""Oracle for the structure-aware layout plan (paper Section 5: the optimisation
problem and Algorithm 1).  TEST INFRASTRUCTURE ONLY - never imported by the product.

Notation follows the paper: tensors t with size e_t (elements), sharding block
("granularity") g_t, u_t = ceil(e_t / g_t) blocks; m devices; uniform per-device
size S; tensor t occupies the contiguous interval [l_t, r_t) = [l_t, l_t + e_t) of
a buffer of m*S elements; device k (0-based here, 1-based in the paper) owns
[k*S, (k+1)*S).

Constraints (Section 5, the unnumbered minimisation problem):
  (C1) r_t - l_t = e_t and r_t <= m*S            (contiguous tensor memory)
  (C2) intervals pairwise disjoint
  (C3) for every k: k*S <= l_t  or  k*S >= r_t  or  (k*S - l_t) = 0 mod g_t
                                                  (non-sharded block)
Balanced load is the uniform S itself.

Readings taken where the paper is silent (listed again in the design notes):
  * u_t = ceil(e_t/g_t): the last block may be short; (C3) is unchanged.
  * S and every l_t are multiples of an alignment: S of g_coll (the collective's
    preferred unit, Algorithm 1 input), l_t of A (tensor-start alignment, A | g_coll).
  * For a FIXED tensor order, CheckValidShard(S) places each tensor at the smallest
    feasible start at or after the previous tensor's end.  Whether a start is
    feasible depends only on (l, e_t, g_t, S), never on other tensors, and padding
    between tensors is free, so by induction this greedy minimises every r_t and
    hence every dp(t, i; S) of Algorithm 1.  dp() below is derived from it.
  * "min{k*g : CheckValidShard(k*g)}" is found by lower-bound bisection on k over
    [1, ceil(total/g)], as the text prescribes ("binary-search"); it is exact where
    feasibility is monotone over multiples of g and otherwise returns some feasible S.
  * g_coll alone is tried as a unit before the first block size (it can only lower S*).
  * The listing forms its units from the ascending block sizes, the text from prefixes of the
    tensors sorted by element count; both families are searched, and every single block size
    on its own (candidate_units).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from math import gcd
from typing import Callable, List, Optional, Sequence, Tuple

BLOCK_1x128 = 0      # 1-D: g = 128 elements;  2-D: g = one row (C elements), 1x128 quant blocks
BLOCK_128x128 = 1    # 2-D only: g = 128 rows (128*C elements), 128x128 quant blocks
BLOCK_WHOLE = 2      # g = e (matrix optimisers: the whole tensor on one device), no quantisation
BLOCK_EXPLICIT = 3   # g given by the caller, no quantisation
BLOCK_32x32 = 4      # 2-D: g = 32 rows (Section 6.3, block-wise 8-bit optimiser state); 1-D: g = 128


def lcm(a: int, b: int) -> int:
    return a // gcd(a, b) * b


def ceil_div(a: int, b: int) -> int:
    return -(-a // b)


def size_and_granularity(rows: int, cols: int, mode: int, g_explicit: int = 0) -> Tuple[int, int]:
    """(e_t, g_t) of one tensor.  cols == 0 means a 1-D tensor of `rows` elements.

    Row-wise RaggedShard (Section 4): the granularity is k whole rows, which is how
    2-D quantisation tiles become contiguous runs (Section 6.3: granularity of 32 rows for
    32x32 blocks; Section 6.4: 128 rows give 128x128 tiles)."""
    if rows <= 0 or cols < 0:
        raise ValueError("empty or negative tensor shape")
    e = rows * cols if cols > 0 else rows
    if mode == BLOCK_1x128:
        g = cols if cols > 0 else 128
    elif mode == BLOCK_128x128:
        if cols == 0:
            raise ValueError("128x128 blocks need a 2-D tensor")
        g = 128 * cols
    elif mode == BLOCK_32x32:
        g = 32 * cols if cols > 0 else 128
    elif mode == BLOCK_WHOLE:
        g = e
    elif mode == BLOCK_EXPLICIT:
        g = g_explicit
    else:
        raise ValueError("unknown block mode")
    if g <= 0:
        raise ValueError("granularity must be positive")
    return e, g


# --------------------------------------------------------------------------------------
# Feasibility of one tensor's start (constraint C3), by definition and in closed form
# --------------------------------------------------------------------------------------

def start_is_feasible(l: int, e: int, g: int, S: int, A: int) -> bool:
    """(C3) written out: every device boundary k*S strictly inside [l, l+e) must fall on a
    block boundary of the tensor; plus the start alignment l = 0 mod A."""
    if l % A != 0:
        return False
    k = l // S + 1
    while k * S < l + e:
        if (k * S - l) % g != 0:
            return False
        k += 1
    return True


def smallest_start_scan(p: int, e: int, g: int, S: int, A: int) -> Optional[int]:
    """Smallest feasible l >= p by trying every aligned candidate.  Feasibility of l and
    of l + S coincide (all boundaries shift together and A | S), so one period suffices."""
    l0 = ceil_div(p, A) * A
    for l in range(l0, l0 + S, A):
        if start_is_feasible(l, e, g, S, A):
            return l
    return None


def smallest_start(p: int, e: int, g: int, S: int, A: int) -> Optional[int]:
    """Smallest feasible l >= p via the paper's three-case analysis (Section 5):
    (1) the tensor lies inside one shard, (2) it straddles exactly one boundary,
    (3) it contains whole shards - possible only if g | S, because two consecutive
    boundaries inside the tensor force S = 0 mod g.  Cross-checked against the scan."""
    l0 = ceil_div(p, A) * A
    B1 = (l0 // S + 1) * S                     # first boundary after l0
    if l0 + e <= B1:                           # case (1) at the earliest aligned slot
        return l0
    if S % g == 0:
        # every boundary is 0 mod g, so l is feasible iff l = 0 mod g (and mod A);
        # anything smaller than that multiple still crosses B1 and is infeasible
        L = lcm(g, A)
        return ceil_div(l0, L) * L
    # g does not divide S: at most ONE boundary B may lie inside the tensor, at
    # l = B - j*g with j >= 1 blocks before it.  A | B, so l = 0 mod A iff st | j.
    st = A // gcd(A, g)
    jmin = max(1, ceil_div(e - S, g))          # the tail must end by B + S

    def straddle(B: int, low: int) -> Optional[int]:
        j = ((B - low) // g) // st * st        # most whole blocks that still start at/after `low`
        return B - j * g if j >= jmin else None

    cand = straddle(B1, l0)                    # case (2) across B1 (B1 - l0 < e, so it does cross)
    if cand is not None:
        return cand
    if e <= S:                                 # case (1), flush at the next boundary
        return B1
    return straddle(B1 + S, B1)                # case (2) across the following boundary; beyond
                                               # that the pattern repeats with period S


StartFn = Callable[[int, int, int, int, int], Optional[int]]


def greedy_layout(tensors: Sequence[Tuple[int, int]], S: int, A: int,
                  start: StartFn = smallest_start) -> Optional[List[int]]:
    """l_t for the given order: each tensor at the smallest feasible start >= end of
    the previous one.  None if some tensor has no feasible start at this S."""
    p = 0
    out = []
    for e, g in tensors:
        l = start(p, e, g, S, A)
        if l is None:
            return None
        out.append(l)
        p = l + e
    return out


def check_valid_shard(tensors: Sequence[Tuple[int, int]], m: int, S: int, A: int,
                      start: StartFn = smallest_start) -> bool:
    """CheckValidShard(S) of Algorithm 1: dp(t_last, u_last; S) <= m, i.e. the greedy
    layout exists and ends within m shards."""
    ls = greedy_layout(tensors, S, A, start)
    if ls is None:
        return False
    if not tensors:
        return True
    return ls[-1] + tensors[-1][0] <= m * S


def dp_value(l_t: int, e: int, g: int, i: int, S: int) -> int:
    """dp(t, i; S): number of device-local shards needed to hold every earlier tensor
    and blocks 0..i (0-based) of tensor t, given t's (minimal) start l_t."""
    end = l_t + min((i + 1) * g, e)
    return ceil_div(end, S)


def dp_segments(tensors: Sequence[Tuple[int, int]], offsets: Sequence[int], S: int):
    """The segment records of CheckValidShard: for each tensor the maximal runs [l, r] of
    block indices with equal dp value (dp is monotone in i, so runs partition [0, u_t))."""
    records = []
    for (e, g), l_t in zip(tensors, offsets):
        u = ceil_div(e, g)
        segs = []
        l = 0
        while l < u:
            v = dp_value(l_t, e, g, l, S)
            # r = max{i : dp(t, i; S) = v}: the last block that still ends within shard v
            r = u - 1 if l_t + e <= v * S else (v * S - l_t) // g - 1
            segs.append((l, r, v))
            l = r + 1
        records.append(segs)
    return records


# --------------------------------------------------------------------------------------
# Outer search of Algorithm 1
# --------------------------------------------------------------------------------------

UNITS_ALL, UNITS_LISTING = 0, 1


def candidate_units(tensors: Sequence[Tuple[int, int]], g_coll: int, units: int = UNITS_ALL) -> List[int]:
    """The units whose multiples are searched.  units = UNITS_LISTING keeps to Algorithm 1 as
    listed (the first family below, g_coll included); the default takes all three.  Algorithm 1's listing and the text around it
    describe two different families; both are taken (every result passes CheckValidShard, so
    more candidates can only lower S*):
      * the listing: g_coll, then the running LCM over the distinct block sizes, ascending;
      * the text: the tensors that can contain a whole shard are the largest ones, so the
        running LCM (from g_coll) over the block sizes of the tensors sorted by element count,
        largest first (equal counts keep the list order) - one unit per prefix;
      * and, since the set of tensors that contain a whole shard may be neither kind of prefix,
        the smallest such sets as well: lcm(g_coll, g) for every distinct block size on its own."""
    found = [g_coll]
    g = g_coll
    for gp in sorted({g_t for _, g_t in tensors}):
        g = lcm(g, gp)
        if g not in found:
            found.append(g)
    if units == UNITS_LISTING:
        return found
    g = g_coll
    for _, gp in sorted(tensors, key=lambda eg: -eg[0]):     # sorted() is stable
        g = lcm(g, gp)
        if g not in found:
            found.append(g)
    for gp in sorted({g_t for _, g_t in tensors}):
        g = lcm(g_coll, gp)
        if g not in found:
            found.append(g)
    return found


def min_feasible_multiple(tensors, m: int, c: int, A: int, start: StartFn = smallest_start) -> int:
    """Lower-bound bisection for min{k*c : CheckValidShard(k*c)}.  k = hi puts every
    tensor (start-aligned) into one shard, which is always feasible."""
    total = sum(ceil_div(e, A) * A for e, _ in tensors)
    lo, hi = 1, max(1, ceil_div(total, c))
    while lo < hi:
        mid = (lo + hi) // 2
        if check_valid_shard(tensors, m, mid * c, A, start):
            hi = mid
        else:
            lo = mid + 1
    return lo * c


def plan_shard_size(tensors: Sequence[Tuple[int, int]], m: int, g_coll: int, A: int,
                    start: StartFn = smallest_start, units: int = UNITS_ALL) -> int:
    """S* of Algorithm 1 for the given tensor order."""
    if m <= 0 or g_coll <= 0 or A <= 0 or g_coll % A != 0 or not tensors:
        raise ValueError("bad plan arguments")
    total = sum(ceil_div(e, A) * A for e, _ in tensors)
    cap = ceil_div(total, g_coll) * g_coll     # one-shard size; larger units cannot win
    best = None
    for c in candidate_units(tensors, g_coll, units):
        if c > cap:
            continue
        s = min_feasible_multiple(tensors, m, c, A, start)
        if best is None or s < best:
            best = s
    return best


# --------------------------------------------------------------------------------------
# The plan of one FSDP unit and the tables derived from it
# --------------------------------------------------------------------------------------

@dataclass
class TensorSpec:
    rows: int
    cols: int            # 0 => 1-D
    mode: int
    g_explicit: int = 0
    e: int = 0
    g: int = 0

    def __post_init__(self):
        self.e, self.g = size_and_granularity(self.rows, self.cols, self.mode, self.g_explicit)

    @property
    def quantised(self) -> bool:
        return self.mode in (BLOCK_1x128, BLOCK_128x128)

    @property
    def nbc(self) -> int:
        """quantisation blocks per row of blocks (1 for 1-D tensors)"""
        return ceil_div(self.cols, 128) if self.cols > 0 else 1

    @property
    def nbr(self) -> int:
        """rows of quantisation blocks"""
        if self.cols == 0:
            return ceil_div(self.rows, 128)
        return ceil_div(self.rows, 128) if self.mode == BLOCK_128x128 else self.rows

    @property
    def num_blocks(self) -> int:
        return self.nbr * self.nbc if self.quantised else 0


@dataclass
class Plan:
    specs: List[TensorSpec]
    m: int
    g_coll: int
    A: int
    S: int = 0
    offsets: List[int] = field(default_factory=list)   # l_t, indexed like specs
    perm: List[int] = field(default_factory=list)      # buffer order: perm[j] = index of the j-th tensor

    def buffer_order(self) -> List[int]:
        return self.perm if self.perm else list(range(len(self.specs)))

    @property
    def total(self) -> int:
        return self.m * self.S

    @property
    def payload(self) -> int:
        return sum(s.e for s in self.specs)

    @property
    def padding(self) -> int:
        return self.total - self.payload

    # --- per-rank segments: the intersection of each tensor with the rank's region
    def rank_segments(self, k: int) -> List[Tuple[int, int, int, int]]:
        """[(t, src_off, dst_off, n)]: n elements of tensor t starting at src_off live at
        offset dst_off of rank k's region."""
        lo, hi = k * self.S, (k + 1) * self.S
        out = []
        for t in self.buffer_order():
            s, l = self.specs[t], self.offsets[t]
            a, b = max(l, lo), min(l + s.e, hi)
            if a < b:
                out.append((t, a - l, a - lo, b - a))
        return out

    # --- scale layout: one flat fp32 array, tensor-major, block-row, block-column
    def scale_bases(self) -> List[int]:
        """First scale of every tensor (indexed like specs) and, last, the total.  The scale
        array follows the buffer: tensors in buffer order."""
        out, acc = [0] * (len(self.specs) + 1), 0
        for t in self.buffer_order():
            out[t] = acc
            acc += self.specs[t].num_blocks
        out[-1] = acc
        return out

    def scale_range(self, k: int) -> Tuple[int, int]:
        """[sb_k, sb_{k+1}): the scales rank k owns.  Whole granules (each = nbc whole
        quantisation blocks) live on one rank, in buffer order, so the range is contiguous."""
        def before(x):
            n = 0
            for s, l in zip(self.specs, self.offsets):
                if not s.quantised:
                    continue
                u = ceil_div(s.e, s.g)
                n += s.nbc * min(u, max(0, ceil_div(x - l, s.g)))
            return n
        return before(k * self.S), before((k + 1) * self.S)


ORDER_DEFAULT = 0      # the order the caller lists the tensors in (the one the paper adopts)
ORDER_BLOCK_SIZE = 1   # stable sort by sharding block size g_t, ascending
ORDER_SHAPE = 2        # stable sort by shape: (element count, rows, cols) ascending
ORDER_BEST = 3         # the three above in turn; smallest S* wins, earlier heuristic on ties


def tensor_order(specs: Sequence[TensorSpec], order: int) -> List[int]:
    """The three tensor orders of Section 5 ("heuristic-guided solution").  The paper names
    them without fixing directions or tie-breaks; this is the reading taken."""
    idx = list(range(len(specs)))
    if order == ORDER_DEFAULT:
        return idx
    if order == ORDER_BLOCK_SIZE:
        return sorted(idx, key=lambda t: specs[t].g)                      # sorted() is stable
    if order == ORDER_SHAPE:
        return sorted(idx, key=lambda t: (specs[t].e, specs[t].rows, specs[t].cols))
    raise ValueError("unknown tensor order")


def make_plan(specs: Sequence[TensorSpec], m: int, align_bytes: int = 16, min_itemsize: int = 1,
              tensor_align: Optional[int] = None, start: StartFn = smallest_start,
              order: int = ORDER_DEFAULT, units: int = UNITS_ALL) -> Plan:
    """plan(): S* by Algorithm 1, then the canonical (earliest-start) layout at S*."""
    if align_bytes % min_itemsize != 0:
        raise ValueError("alignment must be a multiple of the item size")
    g_coll = align_bytes // min_itemsize
    A = g_coll if tensor_align is None else tensor_align
    if order == ORDER_BEST:
        plans = [make_plan(specs, m, align_bytes, min_itemsize, tensor_align, start, o, units)
                 for o in (ORDER_DEFAULT, ORDER_BLOCK_SIZE, ORDER_SHAPE)]
        return min(plans, key=lambda p: p.S)                              # min() keeps the first of equals
    perm = tensor_order(specs, order)
    tensors = [(specs[t].e, specs[t].g) for t in perm]
    S = plan_shard_size(tensors, m, g_coll, A, start, units)
    placed = greedy_layout(tensors, S, A, start)
    assert placed is not None and placed[-1] + tensors[-1][0] <= m * S
    offsets = [0] * len(specs)
    for j, t in enumerate(perm):
        offsets[t] = placed[j]
    return Plan(list(specs), m, g_coll, A, S, offsets, perm)


# --------------------------------------------------------------------------------------
# Invariant checker (constraints C1-C3 + alignment), used on any proposed layout
# --------------------------------------------------------------------------------------

def layout_violations(tensors: Sequence[Tuple[int, int]], offsets: Sequence[int], m: int, S: int,
                      g_coll: int = 1, A: int = 1) -> List[str]:
    """Every way a layout breaks the problem's constraints (empty list = valid)."""
    bad = []
    if S % g_coll != 0:
        bad.append("S not a multiple of g_coll")
    iv = []
    for t, ((e, g), l) in enumerate(zip(tensors, offsets)):
        if l < 0 or l + e > m * S:
            bad.append(f"tensor {t} outside the buffer")
        if l % A != 0:
            bad.append(f"tensor {t} start not aligned")
        for k in range(1, m):
            b = k * S
            if l < b < l + e and (b - l) % g != 0:
                bad.append(f"tensor {t}: boundary of device {k} splits a block")
        iv.append((l, l + e, t))
    iv.sort()
    for (a0, b0, t0), (a1, b1, t1) in zip(iv, iv[1:]):
        if a1 < b0:
            bad.append(f"tensors {t0} and {t1} overlap")
    return bad
