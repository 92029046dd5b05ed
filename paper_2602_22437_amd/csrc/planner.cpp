// Host planner: Algorithm 1 (structure-aware planning for grouped RaggedShard tensors,
// paper Section 5) for a fixed tensor order.
//
// CheckValidShard(S) is evaluated as an earliest-start sweep: whether a start l is
// admissible for tensor t depends on (l, e_t, g_t, S) alone, and padding between tensors
// costs nothing, so taking the smallest admissible start after the previous tensor's end
// minimises every tensor's end and with it dp(t, i; S), the number of device shards used.
// The smallest admissible start comes from the section's three-case analysis (inside one
// shard / across one boundary / containing whole shards) in O(1).
#include <algorithm>
#include <cstdint>
#include <vector>

#include "rs_internal.h"

namespace rs {
namespace {

using i128 = __int128;
constexpr int64_t kLimit = int64_t(1) << 62;

inline int64_t gcd64(int64_t a, int64_t b) {
  while (b != 0) {
    const int64_t r = a % b;
    a = b;
    b = r;
  }
  return a;
}

inline int64_t round_up(int64_t v, int64_t unit) { return (v + unit - 1) / unit * unit; }

}  // namespace

// Smallest l >= p with l = 0 (mod A) such that every rank boundary k*S strictly inside
// [l, l + e) is a multiple of g away from l (the "non-sharded block" constraint).
// Requires A | S.  Returns -1 when no start exists.
int64_t smallest_feasible_start(int64_t p, int64_t e, int64_t g, int64_t S, int64_t A) {
  const int64_t first = round_up(p, A);
  const int64_t next = (first / S + 1) * S;  // boundary closing the shard `first` lies in
  if (first + e <= next) return first;        // case 1: no boundary inside the tensor

  if (S % g == 0) {
    // Boundaries are all congruent mod g, so any number of them may fall inside the tensor
    // (case 3) as long as l itself is a multiple of g; l must also keep the A alignment.
    const i128 unit = i128(g / gcd64(g, A)) * A;
    const i128 v = (i128(first) + unit - 1) / unit * unit;
    return v >= kLimit ? -1 : int64_t(v);
  }

  // g does not divide S: two boundaries inside one tensor would force g | S, so exactly one
  // boundary B may be crossed (case 2), with j >= 1 whole blocks in front of it: l = B - j*g.
  // A | B, hence l stays aligned iff j is a multiple of A / gcd(A, g); the part behind B
  // must end by B + S, which bounds j from below.
  const int64_t j_step = A / gcd64(A, g);
  const int64_t j_need = e > S ? std::max<int64_t>(1, (e - S + g - 1) / g) : 1;
  auto across = [&](int64_t boundary, int64_t not_before) -> int64_t {
    int64_t j = (boundary - not_before) / g;
    j -= j % j_step;
    return j >= j_need ? boundary - j * g : -1;
  };
  const int64_t a = across(next, first);
  if (a >= 0) return a;
  if (e <= S) return next;  // case 1 again: flush against the next boundary
  return across(next + S, next);  // later boundaries repeat this one with period S
}

bool check_valid_shard(const std::vector<TensorHost>& t, int64_t world, int64_t S, int64_t A,
                       std::vector<int64_t>* starts) {
  const i128 room = i128(world) * S;
  int64_t cursor = 0;
  if (starts) starts->assign(t.size(), 0);
  for (size_t i = 0; i < t.size(); ++i) {
    const int64_t l = smallest_feasible_start(cursor, t[i].e, t[i].g, S, A);
    if (l < 0 || i128(l) + t[i].e > room) return false;
    if (starts) (*starts)[i] = l;
    cursor = l + t[i].e;
  }
  return true;
}

int describe_tensors(const rs_tensor_desc* descs, int n, std::vector<TensorHost>* out) {
  out->clear();
  out->reserve(n);
  i128 sum = 0;
  for (int i = 0; i < n; ++i) {
    const rs_tensor_desc& d = descs[i];
    if (d.rows <= 0 || d.cols < 0 || d.reserved != 0) return RS_EINVAL;
    if (d.cols > 0 && d.rows > kLimit / d.cols) return RS_EOVERFLOW;
    if (d.rows >= kLimit || d.cols >= (int64_t(1) << 35)) return RS_EOVERFLOW;  // block counts per row fit 32 bits
    TensorHost h{};
    h.rows = d.rows;
    h.cols = d.cols;
    h.mode = d.block_mode;
    h.e = d.cols > 0 ? d.rows * d.cols : d.rows;
    switch (d.block_mode) {
      case RS_BLOCK_1x128:
        h.g = d.cols > 0 ? d.cols : 128;
        h.quant = true;
        h.nbc = d.cols > 0 ? (d.cols + 127) / 128 : (d.rows + 127) / 128;
        h.nbr = d.cols > 0 ? d.rows : 1;
        break;
      case RS_BLOCK_128x128:
        if (d.cols == 0) return RS_EINVAL;
        h.g = 128 * d.cols;
        h.quant = true;
        h.nbc = (d.cols + 127) / 128;
        h.nbr = (d.rows + 127) / 128;
        break;
      case RS_BLOCK_32x32:
        h.g = d.cols > 0 ? 32 * d.cols : 128;
        break;
      case RS_BLOCK_WHOLE:
        h.g = h.e;
        break;
      case RS_BLOCK_EXPLICIT:
        if (d.g_explicit <= 0) return RS_EINVAL;
        h.g = d.g_explicit;
        break;
      default:
        return RS_EINVAL;
    }
    // 8-bit optimiser-state blocks, the finest that stay whole on a rank: 32x32 tiles where the
    // granularity is whole rows of such tiles; runs of 128 along each row where it is one row,
    // and on 1-D tensors whose granularity is 128
    if (d.cols > 0 && (d.block_mode == RS_BLOCK_32x32 || d.block_mode == RS_BLOCK_128x128)) {
      h.state = true;
      h.sbr = (d.rows + 31) / 32;
      h.sbc = (d.cols + 31) / 32;
    } else if (d.cols > 0 && d.block_mode == RS_BLOCK_1x128) {
      h.state = h.state_runs = true;
      h.sbr = d.rows;
      h.sbc = (d.cols + 127) / 128;
    } else if (d.cols == 0 && (d.block_mode == RS_BLOCK_32x32 || d.block_mode == RS_BLOCK_1x128)) {
      h.state = h.state_runs = true;
      h.sbr = (d.rows + 127) / 128;
      h.sbc = 1;
    }
    h.u = (h.e + h.g - 1) / h.g;
    sum += h.e;
    if (sum >= kLimit) return RS_EOVERFLOW;
    out->push_back(h);
  }
  return RS_OK;
}

// Tensor orders of the heuristic-guided solution (Section 5): the caller's order, ascending
// sharding block size, or ascending shape (element count, rows, cols); stable, so equal keys
// keep the caller's order.
void order_tensors(const std::vector<TensorHost>& t, int order, std::vector<int32_t>* perm) {
  perm->resize(t.size());
  for (size_t i = 0; i < t.size(); ++i) (*perm)[i] = int32_t(i);
  if (order == RS_ORDER_BLOCK_SIZE) {
    std::stable_sort(perm->begin(), perm->end(),
                     [&](int32_t a, int32_t b) { return t[size_t(a)].g < t[size_t(b)].g; });
  } else if (order == RS_ORDER_SHAPE) {
    std::stable_sort(perm->begin(), perm->end(), [&](int32_t a, int32_t b) {
      const TensorHost &x = t[size_t(a)], &y = t[size_t(b)];
      if (x.e != y.e) return x.e < y.e;
      if (x.rows != y.rows) return x.rows < y.rows;
      return x.cols < y.cols;
    });
  }
}

// Outer loop of Algorithm 1: per candidate unit the smallest feasible multiple by lower-bound
// bisection; S* = the minimum.  Three families of units, all starting from g_coll: the listing's
// running LCM over the ascending distinct block sizes, and the text's running LCM over the block
// sizes of the tensors sorted by element count, largest first (the tensors that can contain a
// whole shard), one unit per prefix; and every distinct block size on its own.  Every candidate
// S passes the exact check, so more candidates can only lower S*.
int solve_shard_size(const std::vector<TensorHost>& t, int64_t world, int64_t g_coll, int64_t A,
                     bool listing_only, int64_t* S_out) {
  i128 total = 0;
  for (const TensorHost& h : t) total += round_up(h.e, A);
  if (total >= kLimit) return RS_EOVERFLOW;
  // Everything start-aligned in a single shard is always feasible; a unit beyond that size
  // can only tie or lose.
  const int64_t one_shard = round_up(int64_t(total), g_coll);

  std::vector<int64_t> units{g_coll};
  auto add_family = [&](const std::vector<int64_t>& block_sizes) {
    i128 unit = g_coll;
    for (int64_t g : block_sizes) {
      unit = unit / gcd64(int64_t(unit), g) * g;
      if (unit > one_shard) break;   // the running LCM only grows
      if (std::find(units.begin(), units.end(), int64_t(unit)) == units.end())
        units.push_back(int64_t(unit));
    }
  };
  std::vector<int64_t> sizes;
  for (const TensorHost& h : t) sizes.push_back(h.g);
  std::sort(sizes.begin(), sizes.end());
  sizes.erase(std::unique(sizes.begin(), sizes.end()), sizes.end());
  add_family(sizes);
  if (!listing_only) {
  std::vector<size_t> by_count(t.size());
  for (size_t i = 0; i < t.size(); ++i) by_count[i] = i;
  std::stable_sort(by_count.begin(), by_count.end(),
                   [&](size_t a, size_t b) { return t[a].e > t[b].e; });
  std::vector<int64_t> by_size;
  for (size_t i : by_count) by_size.push_back(t[i].g);
  add_family(by_size);
  // the set of tensors that contain a whole shard may be neither kind of prefix: the smallest
  // such sets as well, every distinct block size on its own
  for (int64_t g : sizes) add_family(std::vector<int64_t>{g});
  }

  int64_t best = -1;
  for (int64_t c : units) {
    int64_t lo = 1, hi = std::max<int64_t>(1, (int64_t(total) + c - 1) / c);
    while (lo < hi) {
      const int64_t mid = lo + (hi - lo) / 2;
      if (i128(mid) * c < kLimit && check_valid_shard(t, world, mid * c, A, nullptr))
        hi = mid;
      else
        lo = mid + 1;
    }
    if (i128(lo) * c >= kLimit) continue;
    const int64_t cand = lo * c;
    if (best < 0 || cand < best) best = cand;
  }
  if (best < 0 || i128(best) * world >= kLimit) return RS_EOVERFLOW;
  *S_out = best;
  return RS_OK;
}

// Composition with an even Shard(dim > 0) (Section 4): ragged boundaries must leave dimension
// `dim` whole, i.e. fall on multiples of the extent of dimensions dim.. of the row-major tensor;
// the granularity is the least common multiple of that extent and the caller's granularity.
int shard_dim_granularity(const int64_t* shape, int ndim, int dim, int64_t g_user, int64_t* g_out) {
  if (!shape || !g_out || ndim < 2 || dim <= 0 || dim >= ndim || g_user <= 0) return RS_EINVAL;
  i128 plane = 1, elems = 1;
  for (int d = ndim - 1; d >= 0; --d) {
    if (shape[d] <= 0) return RS_EINVAL;
    elems *= shape[d];
    if (elems >= kLimit) return RS_EOVERFLOW;
    if (d >= dim) plane = elems;
  }
  const i128 g = plane / gcd64(int64_t(plane), g_user) * g_user;
  if (g >= kLimit) return RS_EOVERFLOW;
  *g_out = int64_t(g);
  return RS_OK;
}

// SelectRoot of Algorithm 2 as longest-processing-time-first list scheduling.  The cost of an
// R x C matrix is one quintic Newton-Schulz iteration in units of two flops: a*a*(2b + a) with
// a = min(R, C), b = max(R, C) (Gram matrix, its square, the update).  Costs stay below 2^95 and
// their sums below 2^126, so 128-bit integers are exact.
void select_roots(const std::vector<TensorHost>& t, int world, int32_t* roots, double* loads) {
  using u128 = unsigned __int128;
  std::vector<u128> cost(t.size(), 0), acc(size_t(world), 0);
  std::vector<int32_t> mats;
  for (size_t i = 0; i < t.size(); ++i) {
    roots[i] = -1;
    if (t[i].cols == 0) continue;
    const u128 a = u128(std::min(t[i].rows, t[i].cols)), b = u128(std::max(t[i].rows, t[i].cols));
    cost[i] = a * a * (2 * b + a);
    mats.push_back(int32_t(i));
  }
  std::stable_sort(mats.begin(), mats.end(),
                   [&](int32_t x, int32_t y) { return cost[size_t(x)] > cost[size_t(y)]; });
  for (int32_t i : mats) {
    size_t k = 0;
    for (size_t d = 1; d < acc.size(); ++d)
      if (acc[d] < acc[k]) k = d;
    roots[size_t(i)] = int32_t(k);
    acc[k] += cost[size_t(i)];
  }
  if (loads)
    for (size_t d = 0; d < acc.size(); ++d) loads[d] = double(acc[d]);
}

// The buffer of a group placed RaggedShard(r_t): device k's region holds the tensors rooted at
// k in the caller's order, starts aligned to A; S = the largest region rounded up to g_coll.
// `t` is in the caller's order; perm receives the buffer order, starts the offsets in that order.
int rooted_layout(const std::vector<TensorHost>& t, int64_t world, int64_t g_coll, int64_t A,
                  const int32_t* roots, std::vector<int32_t>* perm, std::vector<int64_t>* starts,
                  int64_t* S_out) {
  std::vector<i128> extent(size_t(world), 0);
  std::vector<i128> rel(t.size(), 0);
  i128 longest = 0;
  for (size_t i = 0; i < t.size(); ++i) {
    if (roots[i] < 0 || roots[i] >= world) return RS_EINVAL;
    i128& x = extent[size_t(roots[i])];
    rel[i] = (x + A - 1) / A * A;
    x = rel[i] + t[i].e;
    longest = std::max(longest, x);
  }
  const i128 S = (longest + g_coll - 1) / g_coll * g_coll;
  if (S * world >= kLimit) return RS_EOVERFLOW;
  perm->resize(t.size());
  for (size_t i = 0; i < t.size(); ++i) (*perm)[i] = int32_t(i);
  std::stable_sort(perm->begin(), perm->end(),
                   [&](int32_t x, int32_t y) { return roots[x] < roots[y]; });
  starts->resize(t.size());
  for (size_t j = 0; j < t.size(); ++j) {
    const size_t i = size_t((*perm)[j]);
    (*starts)[j] = int64_t(S * roots[i] + rel[i]);
  }
  *S_out = int64_t(S);
  return RS_OK;
}

}  // namespace rs
