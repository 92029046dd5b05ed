// Internal structures shared by the host planner, the table builder and the HIP kernels.
#pragma once
#include <cstdint>
#include <vector>

#include "raggedshard.h"

namespace rs {

// Tile-table granule: the DBuffer region of every rank is cut into granules of this many
// elements; the table gives, per granule, the first tensor that ends after the granule's start.
constexpr int kGranule = 2048;
// gran_first entries carry this flag when the granule lies wholly inside the tensor they name:
// a workgroup then knows all of its elements are payload without reading the tensor's record.
constexpr int32_t kGranWhole = int32_t(1) << 30;
// A quantisation work item covers at most this many "row slots" of 128 elements:
// one 128x128 tile, or 128 consecutive 1x128 blocks.
constexpr int kItemSlots = 128;
// Optimiser-state work items: 32 rows x kStateCols columns of a 2-D tensor (one row of
// kStateCols / 32 state tiles), or kStateRuns consecutive 128-element runs of a 1-D tensor.
constexpr int kStateCols = 256;
constexpr int kStateRuns = 64;
// A zero-fill item clears at most this many code bytes.
constexpr int kFillElems = 32768;

enum : int32_t {
  kFlagTile = 1,     // 128x128 tiles (else 1x128 runs)
  kFlagQuant = 2,    // tensor has FP8 blocks
  kFlagVec = 4,      // every row slot starts 8-element aligned in the buffer (16-byte bf16 vectors)
  kFlagContig = 8,   // 1x128 blocks are back to back in memory (1-D, or C % 128 == 0)
  kFlagState = 16,   // tensor has 8-bit optimiser-state blocks
  kFlagVec4 = 32,    // every row starts 4-element aligned in the buffer (16-byte fp32 vectors)
  kFlagStateRuns = 64  // state blocks are runs of 128 along each row (1-D tensors, one-row granularity)
};

// Per-tensor record on the device (64 bytes).
struct TensorDev {
  int64_t ell;         // l_t: first element in the buffer
  int64_t e;           // elements
  int64_t scale_base;  // first scale index
  int64_t rows;        // R (1 for 1-D tensors)
  int64_t cols;        // C (n for 1-D tensors)
  int32_t nbc;         // quantisation blocks per row of blocks
  int32_t flags;
  int64_t state_base;  // first optimiser-state block
  int32_t sbc;         // state blocks per row of state blocks (2-D)
  int32_t reserved;
};

// One workgroup's worth of block_quant or optimiser-state work (16 bytes).
struct Item {
  int64_t first;   // tile: block row br;  runs: first block index;  fill: buffer element offset
  int32_t tensor;  // -1 marks a zero-fill item
  int32_t count;   // tile: block column bc;  runs: blocks in this item (<= kItemSlots);  fill: elements
                   // state items: first = row of 32x32 tiles / first run (tensor-wide run index);
                   //              count = column strip / runs in this item (<= kStateRuns)
};

// A quantisation work item (48 bytes): the Item fields plus what lets a workgroup start loading
// without reading the tensor's record first (one table read instead of two dependent ones).
struct alignas(16) QItem {
  int64_t first;   // as Item
  int32_t tensor;  // -1 marks a zero-fill item
  int32_t count;   // as Item
  int64_t elem;    // buffer element of the item's first element (tile: its top-left corner)
  int64_t scale;   // index of the item's first scale in the unit's scale array
  int32_t pitch;   // tile: elements from one row to the next; runs: 128
  int16_t rows;    // tile: rows that exist (1..128); runs: blocks in the item
  int16_t cols;    // tile: columns that exist (1..128); runs: 128
  int32_t lean;    // non-zero: every row piece is 16-byte structured and a whole number of 8-element
                   // groups, so the kernel needs nothing but this record.  1: a tile of any extent;
                   // 2: 128 full back-to-back runs of 128
  int32_t reserved;
};
static_assert(sizeof(QItem) == 48, "three 16-byte loads");

// A granule that holds payload, with the first tensor that ends after its start: what a copy
// workgroup needs to find its work in one table read (8 bytes).
struct alignas(8) GranRef {
  int32_t gid;    // rank * granules_per_rank + index within the rank
  int32_t first;  // gran_first[gid]
};

struct TensorHost {
  int64_t rows, cols;  // as described by the caller (cols == 0: 1-D)
  int32_t mode;
  int64_t e, g, u;     // elements, granularity, ceil(e/g)
  int64_t ell;         // planned start
  int64_t nbr, nbc;    // FP8 block grid (0 x 0 when not quantised)
  int64_t scale_base;
  bool quant;
  bool state;          // 8-bit optimiser-state blocks are defined (and whole on a rank)
  bool state_runs;     // they are runs of 128 along each row (else 32x32 tiles)
  int64_t sbr, sbc;    // state block grid: rows of blocks x blocks per row
  int64_t state_base;
};

struct HostTables {
  std::vector<TensorDev> tensors;
  std::vector<int32_t> gran_first;   // world * granules_per_rank; tensor index, + kGranWhole
  int64_t granules_per_rank = 0;
  std::vector<QItem> items;          // rank-major
  std::vector<int64_t> item_begin;   // world + 1
  // granules that hold at least one payload element (ids = rank * granules_per_rank + index):
  // the unpack kernels launch workgroups for these only and never visit pure padding
  std::vector<GranRef> payload_gran;
  std::vector<int32_t> padding_gran;   // the rest: granules ragged_pack only has to zero
  int64_t n_payload_gran = 0, n_padding_gran = 0;
  std::vector<Item> state_items;            // rank-major; empty unless every tensor has state blocks
  std::vector<int64_t> state_item_begin;    // world + 1
};

struct DeviceTables {
  int device = -1;
  TensorDev* tensors = nullptr;
  int32_t* gran_first = nullptr;
  QItem* items = nullptr;
  GranRef* payload_gran = nullptr;
  int32_t* padding_gran = nullptr;
  Item* state_items = nullptr;
};

// ---- planner (planner.cpp) ----
int64_t smallest_feasible_start(int64_t p, int64_t e, int64_t g, int64_t S, int64_t A);
bool check_valid_shard(const std::vector<TensorHost>& t, int64_t world, int64_t S, int64_t A,
                       std::vector<int64_t>* starts);
int describe_tensors(const rs_tensor_desc* descs, int n, std::vector<TensorHost>* out);
// listing_only: candidate units restricted to Algorithm 1's listing (plus g_coll)
int solve_shard_size(const std::vector<TensorHost>& t, int64_t world, int64_t g_coll, int64_t A,
                     bool listing_only, int64_t* S_out);
void order_tensors(const std::vector<TensorHost>& t, int order, std::vector<int32_t>* perm);
int shard_dim_granularity(const int64_t* shape, int ndim, int dim, int64_t g_user, int64_t* g_out);
void select_roots(const std::vector<TensorHost>& t, int world, int32_t* roots, double* loads);
int rooted_layout(const std::vector<TensorHost>& t, int64_t world, int64_t g_coll, int64_t A,
                  const int32_t* roots, std::vector<int32_t>* perm, std::vector<int64_t>* starts,
                  int64_t* S_out);

// ---- derived tables (tables.cpp) ----
void build_host_tables(const std::vector<TensorHost>& t, int64_t world, int64_t S, bool all_quant,
                       bool all_state, HostTables* out);

}  // namespace rs

struct rs_plan {
  std::vector<rs::TensorHost> t;   // in BUFFER order (increasing l_t)
  std::vector<int32_t> orig;       // orig[j] = caller's index of the j-th tensor in the buffer
  int64_t world = 0, g_coll = 0, A = 0, S = 0, payload = 0, num_scales = 0;
  bool all_quant = false;
  std::vector<int64_t> scale_begin;  // world + 1: first scale of every rank
  bool all_state = false;            // every tensor has 8-bit optimiser-state blocks
  int64_t num_state_blocks = 0;
  std::vector<int64_t> state_begin;  // world + 1: first state block of every rank
  rs::HostTables host;
  rs::DeviceTables dev;
};

struct rs_tensor_table {
  const rs_plan* owner = nullptr;  // tables are valid for the plan they were made for only
  int device = -1;
  int n = 0;
  unsigned low_bits = 0;  // OR of the low four address bits of all pointers
  void** ptrs = nullptr;  // device array of n pointers
};

struct rs_shard_batch {
  const rs_plan* owner = nullptr;
  int rank = 0;
  int count = 0;
  void** ptrs = nullptr;  // device array: count shards, count code buffers, count scale slices
};

struct rs_partials_batch {
  const rs_plan* owner = nullptr;
  int rank = 0;
  int count = 0;
  int64_t row_stride = 0;
  void** ptrs = nullptr;  // device array: count partial buffers, count outputs
};

struct rs_adam8_batch {
  const rs_plan* owner = nullptr;
  int rank = 0;
  int count = 0;
  void** ptrs = nullptr;  // device array: count each of grad, master, param, m codes, v codes, m absmax, v absmax
};
