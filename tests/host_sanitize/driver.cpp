// Host-only driver for the planner and the table builder, compiled with AddressSanitizer and
// UndefinedBehaviorSanitizer by tests/test_host_sanitize.py: random units are planned, their
// device tables are built on the host, and every index the kernels would follow is checked
// against the buffer and tensor bounds.  Exits non-zero on the first violation.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#include "rs_internal.h"

namespace {

uint64_t state = 0x9E3779B97F4A7C15ull;
uint64_t next() {
  state ^= state << 13;
  state ^= state >> 7;
  state ^= state << 17;
  return state;
}
int64_t pick(int64_t lo, int64_t hi) { return lo + int64_t(next() % uint64_t(hi - lo + 1)); }

#define REQUIRE(cond)                                                          \
  do {                                                                         \
    if (!(cond)) {                                                             \
      std::printf("violation at line %d: %s (case %d)\n", __LINE__, #cond, c); \
      return 1;                                                                \
    }                                                                          \
  } while (0)

}  // namespace

int main(int argc, char** argv) {
  const int cases = argc > 1 ? std::atoi(argv[1]) : 400;
  const int64_t widths[] = {8, 24, 30, 32, 40, 100, 128, 130, 136, 256, 300, 1100};
  for (int c = 0; c < cases; ++c) {
    const int n = int(pick(1, 7));
    const bool state_unit = c % 3 == 0;   // every third unit: only tensors that carry 8-bit state
    std::vector<rs_tensor_desc> descs;
    for (int i = 0; i < n; ++i) {
      rs_tensor_desc d{};
      const int kind = int(pick(0, 9));
      if (state_unit) {
        if (kind < 3) {
          d.rows = pick(1, 3000);
          d.block_mode = kind == 0 ? RS_BLOCK_1x128 : RS_BLOCK_32x32;
        } else if (kind == 3) {
          d.rows = pick(1, 90);
          d.cols = widths[pick(0, 11)];
          d.block_mode = RS_BLOCK_1x128;
        } else {
          d.rows = pick(1, 300);
          d.cols = widths[pick(0, 11)];
          d.block_mode = kind < 8 ? RS_BLOCK_32x32 : RS_BLOCK_128x128;
        }
      } else if (kind < 2) {
        d.rows = pick(1, 3000);
        d.block_mode = RS_BLOCK_1x128;
      } else if (kind < 6) {
        d.rows = pick(1, 400);
        d.cols = widths[pick(0, 11)];
        d.block_mode = RS_BLOCK_128x128;
      } else if (kind < 8) {
        d.rows = pick(1, 60);
        d.cols = widths[pick(0, 11)];
        d.block_mode = RS_BLOCK_1x128;
      } else if (kind < 9) {
        d.rows = pick(1, 50);
        d.cols = pick(1, 50);
        d.block_mode = RS_BLOCK_WHOLE;
      } else {
        d.rows = pick(1, 50);
        d.cols = pick(1, 50);
        d.block_mode = RS_BLOCK_EXPLICIT;
        d.g_explicit = pick(1, 64);
      }
      descs.push_back(d);
    }
    const int64_t worlds[] = {1, 2, 3, 4, 7, 8, 16, 33, 128};
    const int64_t world = worlds[pick(0, 8)];
    const int64_t g_coll = (c % 5 == 4) ? 8 : 16;
    const int64_t A = (c % 7 == 6) ? 1 : g_coll;

    std::vector<rs::TensorHost> t;
    REQUIRE(rs::describe_tensors(descs.data(), n, &t) == RS_OK);
    int64_t S = 0;
    std::vector<int64_t> starts;
    if (c % 4 == 1) {
      // every tensor whole on a device of its own choosing; some devices stay empty
      std::vector<int32_t> roots, perm;
      for (int i = 0; i < n; ++i) roots.push_back(int32_t(pick(0, world - 1)));
      REQUIRE(rs::rooted_layout(t, world, g_coll, A, roots.data(), &perm, &starts, &S) == RS_OK);
      std::vector<rs::TensorHost> placed;
      for (size_t j = 0; j < perm.size(); ++j) {
        placed.push_back(t[size_t(perm[j])]);
        const int64_t k = roots[size_t(perm[j])];
        REQUIRE(starts[j] >= k * S && starts[j] + placed.back().e <= (k + 1) * S);
      }
      t = placed;
      std::vector<int32_t> lpt(size_t(n), 0);
      std::vector<double> loads(size_t(world), 0.0);
      rs::select_roots(t, int(world), lpt.data(), loads.data());
      for (int i = 0; i < n; ++i) REQUIRE(t[size_t(i)].cols == 0 ? lpt[size_t(i)] == -1 : (lpt[size_t(i)] >= 0 && lpt[size_t(i)] < world));
    } else {
      REQUIRE(rs::solve_shard_size(t, world, g_coll, A, false, &S) == RS_OK);
      int64_t S_listing = 0;   // Algorithm 1 as listed searches a subset of the units: never better
      REQUIRE(rs::solve_shard_size(t, world, g_coll, A, true, &S_listing) == RS_OK && S_listing >= S);
      REQUIRE(rs::check_valid_shard(t, world, S, A, &starts));
    }
    REQUIRE(S > 0 && S % g_coll == 0);
    bool all_quant = true, all_state = true;
    int64_t sb = 0, stb = 0, prev_end = 0;
    for (size_t i = 0; i < t.size(); ++i) {
      t[i].ell = starts[i];
      REQUIRE(starts[i] >= prev_end && starts[i] % A == 0);
      prev_end = starts[i] + t[i].e;
      // no block is cut by a rank boundary
      for (int64_t k = starts[i] / S + 1; k * S < prev_end; ++k) REQUIRE((k * S - starts[i]) % t[i].g == 0);
      t[i].scale_base = sb;
      sb += t[i].nbr * t[i].nbc;
      t[i].state_base = stb;
      stb += t[i].sbr * t[i].sbc;
      all_quant = all_quant && t[i].quant;
      all_state = all_state && t[i].state;
    }
    REQUIRE(prev_end <= world * S);
    if (state_unit) REQUIRE(all_state);

    rs::HostTables h;
    rs::build_host_tables(t, world, S, all_quant, all_state, &h);
    const int64_t gpr = h.granules_per_rank;
    REQUIRE(gpr == (S + rs::kGranule - 1) / rs::kGranule);
    REQUIRE(int64_t(h.gran_first.size()) == world * gpr);
    REQUIRE(h.n_payload_gran + h.n_padding_gran == world * gpr);
    for (int64_t k = 0; k < world; ++k)
      for (int64_t j = 0; j < gpr; ++j) {
        const int32_t entry = h.gran_first[size_t(k * gpr + j)];
        const int32_t f = entry & ~rs::kGranWhole;
        REQUIRE(f >= 0 && f <= n);
        const int64_t start = k * S + j * rs::kGranule;
        const int64_t stop = std::min(start + rs::kGranule, (k + 1) * S);
        const bool whole = f < n && t[size_t(f)].ell <= start && stop <= t[size_t(f)].ell + t[size_t(f)].e;
        REQUIRE(whole == ((entry & rs::kGranWhole) != 0));
        if (f < n) REQUIRE(t[size_t(f)].ell + t[size_t(f)].e > start);
        if (f > 0) REQUIRE(t[size_t(f - 1)].ell + t[size_t(f - 1)].e <= start);
      }
    // quantisation items: inside their tensor and their rank; fills inside the rank's padding
    if (all_quant) {
      REQUIRE(int64_t(h.item_begin.size()) == world + 1);
      std::vector<int64_t> covered(size_t(world), 0);
      for (int64_t k = 0; k < world; ++k)
        for (int64_t q = h.item_begin[size_t(k)]; q < h.item_begin[size_t(k) + 1]; ++q) {
          const rs::QItem& it = h.items[size_t(q)];
          if (it.tensor < 0) {
            REQUIRE(it.first >= k * S && it.first + it.count <= (k + 1) * S && it.count > 0);
            covered[size_t(k)] += it.count;
            continue;
          }
          REQUIRE(it.tensor < n);
          const rs::TensorHost& x = t[size_t(it.tensor)];
          int64_t lo, hi;   // element range of the item inside the tensor
          if (x.mode == RS_BLOCK_128x128) {
            REQUIRE(it.first >= 0 && it.first < x.nbr && it.count >= 0 && it.count < x.nbc);
            lo = it.first * 128 * x.cols;
            hi = std::min(x.rows, (it.first + 1) * 128) * x.cols;
          } else if (x.cols > 0) {
            REQUIRE(it.count > 0 && it.count <= rs::kItemSlots && it.first + it.count <= x.nbr * x.nbc);
            lo = it.first / x.nbc * x.cols;
            hi = ((it.first + it.count - 1) / x.nbc + 1) * x.cols;
          } else {
            REQUIRE(it.count > 0 && it.count <= rs::kItemSlots);
            lo = it.first * 128;
            hi = std::min(x.e, (it.first + it.count) * 128);
          }
          REQUIRE(lo >= 0 && hi <= x.e && lo < hi);
          REQUIRE(x.ell + lo >= k * S && x.ell + hi <= (k + 1) * S);
          // what the table-free path of the kernel goes by: every 16-byte access it derives from
          // the record alone lies inside the tensor (hence the rank) and is 8-element aligned
          if (it.lean == 1) {
            REQUIRE(x.mode == RS_BLOCK_128x128 && it.pitch == x.cols && x.ell % 8 == 0 && x.cols % 8 == 0);
            REQUIRE(it.rows >= 1 && it.rows <= 128 && it.cols >= 8 && it.cols <= 128 && it.cols % 8 == 0);
            REQUIRE(it.elem == x.ell + it.first * 128 * x.cols + int64_t(it.count) * 128);
            REQUIRE(it.first * 128 + it.rows <= x.rows && int64_t(it.count) * 128 + it.cols <= x.cols);
            REQUIRE(it.rows == 128 || it.first * 128 + it.rows == x.rows);
            REQUIRE(it.cols == 128 || int64_t(it.count) * 128 + it.cols == x.cols);
            REQUIRE(it.scale == x.scale_base + it.first * x.nbc + it.count);
            const int64_t last = it.elem + int64_t(it.rows - 1) * it.pitch + it.cols;   // one past the end
            REQUIRE(it.elem % 8 == 0 && last <= x.ell + x.e);
          } else if (it.lean == 2) {
            REQUIRE(x.mode != RS_BLOCK_128x128 && it.pitch == 128 && it.rows == 128 && it.cols == 128);
            REQUIRE(x.cols == 0 || x.cols % 128 == 0);
            REQUIRE(it.elem == x.ell + it.first * 128 && it.elem % 8 == 0);
            REQUIRE(it.elem + 128 * 128 <= x.ell + x.e && it.count == rs::kItemSlots);
            REQUIRE(it.scale == x.scale_base + it.first);
          } else {
            REQUIRE(it.lean == 0);
          }
        }
      int64_t padding = world * S;
      for (const rs::TensorHost& x : t) padding -= x.e;
      int64_t filled = 0;
      for (int64_t v : covered) filled += v;
      REQUIRE(filled == padding);
    }
    // optimiser-state items: every state block exactly once, inside its rank
    if (all_state) {
      std::vector<int> seen(size_t(stb), 0);
      for (int64_t k = 0; k < world; ++k)
        for (int64_t q = h.state_item_begin[size_t(k)]; q < h.state_item_begin[size_t(k) + 1]; ++q) {
          const rs::Item& it = h.state_items[size_t(q)];
          REQUIRE(it.tensor >= 0 && it.tensor < n);
          const rs::TensorHost& x = t[size_t(it.tensor)];
          if (!x.state_runs) {
            REQUIRE(it.first >= 0 && it.first < x.sbr);
            const int64_t c0 = int64_t(it.count) * rs::kStateCols;
            REQUIRE(c0 < x.cols);
            const int64_t r0 = it.first * 32, r1 = std::min(x.rows, r0 + 32);
            REQUIRE(x.ell + r0 * x.cols >= k * S && x.ell + r1 * x.cols <= (k + 1) * S);
            for (int64_t bc = c0 / 32; bc < std::min<int64_t>(x.sbc, c0 / 32 + rs::kStateCols / 32); ++bc)
              ++seen[size_t(x.state_base + it.first * x.sbc + bc)];
          } else {
            REQUIRE(it.count > 0 && it.count <= rs::kStateRuns && it.first >= 0);
            REQUIRE(it.first + it.count <= x.sbr * x.sbc);
            for (int64_t r = it.first; r < it.first + it.count; ++r) {
              // first and last element of run r
              int64_t lo, hi;
              if (x.cols > 0) {
                const int64_t row = r / x.sbc, bc = r % x.sbc;
                lo = row * x.cols + bc * 128;
                hi = row * x.cols + std::min(x.cols, (bc + 1) * 128);
              } else {
                lo = r * 128;
                hi = std::min(x.e, (r + 1) * 128);
              }
              REQUIRE(lo < hi && x.ell + lo >= k * S && x.ell + hi <= (k + 1) * S);
              ++seen[size_t(x.state_base + r)];
            }
          }
        }
      for (int v : seen) REQUIRE(v == 1);
    }
  }
  std::printf("ok: %d units\n", cases);
  return 0;
}
