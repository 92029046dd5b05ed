// Host construction of the device tables derived from a plan: the per-tensor records, the
// granule -> first-tensor table that lets every workgroup find its tensors with one load, and
// the per-rank work items of block_quant / dequant_unpack.
#include <algorithm>

#include "rs_internal.h"

namespace rs {

namespace {

void add_fill(std::vector<QItem>* items, int64_t from, int64_t to) {
  for (int64_t d = from; d < to; d += kFillElems) {
    QItem it{};
    it.first = d;
    it.tensor = -1;
    it.count = int32_t(std::min<int64_t>(kFillElems, to - d));
    items->push_back(it);
  }
}

}  // namespace

void build_host_tables(const std::vector<TensorHost>& t, int64_t world, int64_t S, bool all_quant,
                       bool all_state, HostTables* out) {
  const int n = int(t.size());
  out->tensors.resize(n);
  for (int i = 0; i < n; ++i) {
    const TensorHost& h = t[i];
    TensorDev d{};
    d.ell = h.ell;
    d.e = h.e;
    d.scale_base = h.scale_base;
    d.rows = h.cols > 0 ? h.rows : 1;
    d.cols = h.cols > 0 ? h.cols : h.rows;
    d.nbc = int32_t(h.nbc);
    int32_t f = 0;
    if (h.quant) f |= kFlagQuant;
    if (h.mode == RS_BLOCK_128x128) f |= kFlagTile;
    const bool one_d = h.cols == 0;
    if (h.ell % 8 == 0 && (one_d || d.cols % 8 == 0)) f |= kFlagVec;
    if (one_d || d.cols % 128 == 0) f |= kFlagContig;
    if (h.state) f |= kFlagState;
    if (h.ell % 4 == 0 && (one_d || d.cols % 4 == 0)) f |= kFlagVec4;
    if (h.state_runs) f |= kFlagStateRuns;
    d.flags = f;
    d.state_base = h.state_base;
    d.sbc = int32_t(h.sbc);
    out->tensors[i] = d;
  }

  // granule table: tensors are in increasing buffer order, so one forward sweep suffices
  const int64_t gpr = (S + kGranule - 1) / kGranule;
  out->granules_per_rank = gpr;
  out->gran_first.resize(size_t(world * gpr));
  int cur = 0;
  for (int64_t k = 0; k < world; ++k) {
    for (int64_t j = 0; j < gpr; ++j) {
      const int64_t start = k * S + j * kGranule;
      while (cur < n && t[cur].ell + t[cur].e <= start) ++cur;
      out->gran_first[size_t(k * gpr + j)] = cur;
    }
  }

  // payload list: a granule holds payload iff its first not-yet-ended tensor starts before its end
  out->payload_gran.clear();
  out->padding_gran.clear();
  for (int64_t k = 0; k < world; ++k) {
    for (int64_t j = 0; j < gpr; ++j) {
      const int32_t f = out->gran_first[size_t(k * gpr + j)];
      const int64_t start = k * S + j * kGranule;
      const int64_t stop = std::min(start + kGranule, (k + 1) * S);
      if (f >= n || t[f].ell >= stop) {
        out->padding_gran.push_back(int32_t(k * gpr + j));
        continue;
      }
      out->payload_gran.push_back(GranRef{int32_t(k * gpr + j), f});
      if (t[f].ell <= start && stop <= t[f].ell + t[f].e) out->gran_first[size_t(k * gpr + j)] = f | kGranWhole;
    }
  }
  out->n_payload_gran = int64_t(out->payload_gran.size());
  out->n_padding_gran = int64_t(out->padding_gran.size());

  // optimiser-state work items, rank by rank in buffer order: a rank's part of a tensor is a
  // run of whole granules, hence of whole rows of state tiles (or whole runs)
  out->state_items.clear();
  out->state_item_begin.assign(size_t(world + 1), 0);
  if (all_state) {
    int first = 0;
    for (int64_t k = 0; k < world; ++k) {
      out->state_item_begin[size_t(k)] = int64_t(out->state_items.size());
      const int64_t lo = k * S, hi = lo + S;
      while (first < n && t[first].ell + t[first].e <= lo) ++first;
      for (int i = first; i < n && t[i].ell < hi; ++i) {
        const TensorHost& h = t[i];
        const int64_t a = std::max(h.ell, lo) - h.ell, b = std::min(h.ell + h.e, hi) - h.ell;
        if (!h.state_runs) {
          const int64_t br_a = a / h.cols / 32, br_b = (b / h.cols + 31) / 32;
          const int64_t strips = (h.cols + kStateCols - 1) / kStateCols;
          for (int64_t br = br_a; br < br_b; ++br)
            for (int64_t cs = 0; cs < strips; ++cs) {
              Item it{};
              it.first = br;
              it.tensor = i;
              it.count = int32_t(cs);
              out->state_items.push_back(it);
            }
        } else {
          // runs of the rank: whole rows of runs (2-D), or runs of a 1-D tensor
          const int64_t q_a = h.cols > 0 ? a / h.cols * h.sbc : a / 128;
          const int64_t q_b = h.cols > 0 ? b / h.cols * h.sbc : (b + 127) / 128;
          for (int64_t q = q_a; q < q_b; q += kStateRuns) {
            Item it{};
            it.first = q;
            it.tensor = i;
            it.count = int32_t(std::min<int64_t>(kStateRuns, q_b - q));
            out->state_items.push_back(it);
          }
        }
      }
    }
    out->state_item_begin[size_t(world)] = int64_t(out->state_items.size());
  }

  // quantisation work items, rank by rank in buffer order, zero-fill items for every gap
  out->items.clear();
  out->item_begin.assign(size_t(world + 1), 0);
  if (!all_quant) return;
  int ti = 0;
  for (int64_t k = 0; k < world; ++k) {
    out->item_begin[size_t(k)] = int64_t(out->items.size());
    const int64_t lo = k * S, hi = lo + S;
    int64_t cursor = lo;
    while (ti < n && t[ti].ell + t[ti].e <= lo) ++ti;
    for (int i = ti; i < n && t[i].ell < hi; ++i) {
      const TensorHost& h = t[i];
      const int64_t a = std::max(h.ell, lo), b = std::min(h.ell + h.e, hi);
      if (a > cursor) add_fill(&out->items, cursor, a);
      cursor = b;
      const int64_t src_a = a - h.ell, src_b = b - h.ell;  // whole granules by construction
      if (h.mode == RS_BLOCK_128x128) {
        const int64_t br_a = src_a / h.g, br_b = (src_b + h.g - 1) / h.g;
        const bool vec = h.ell % 8 == 0 && h.cols % 8 == 0 && h.cols < (int64_t(1) << 31);
        for (int64_t br = br_a; br < br_b; ++br)
          for (int64_t bc = 0; bc < h.nbc; ++bc) {
            QItem it{};
            it.first = br;
            it.count = int32_t(bc);
            it.tensor = i;
            it.elem = h.ell + br * 128 * h.cols + bc * 128;
            it.scale = h.scale_base + br * h.nbc + bc;
            it.pitch = int32_t(std::min<int64_t>(h.cols, 0x7fffffff));
            it.rows = int16_t(std::min<int64_t>(128, h.rows - br * 128));
            it.cols = int16_t(std::min<int64_t>(128, h.cols - bc * 128));
            it.lean = vec ? 1 : 0;
            out->items.push_back(it);
          }
      } else {
        int64_t blk_a, blk_b;
        if (h.cols > 0) {  // one granule = one row = nbc blocks
          blk_a = src_a / h.cols * h.nbc;
          blk_b = src_b / h.cols * h.nbc;
        } else {           // one granule = one block of 128
          blk_a = src_a / 128;
          blk_b = (src_b + 127) / 128;
        }
        const bool contig = h.cols == 0 || h.cols % 128 == 0;
        for (int64_t q = blk_a; q < blk_b; q += kItemSlots) {
          QItem it{};
          it.first = q;
          it.tensor = i;
          it.count = int32_t(std::min<int64_t>(kItemSlots, blk_b - q));
          it.elem = h.ell + q * 128;              // meaningful for back-to-back blocks only
          it.scale = h.scale_base + q;
          it.pitch = 128;
          it.rows = int16_t(it.count);
          it.cols = 128;
          it.lean = (contig && h.ell % 8 == 0 && it.count == kItemSlots && (q + kItemSlots) * 128 <= h.e) ? 2 : 0;
          out->items.push_back(it);
        }
      }
    }
    if (cursor < hi) add_fill(&out->items, cursor, hi);
  }
  out->item_begin[size_t(world)] = int64_t(out->items.size());
}

}  // namespace rs
