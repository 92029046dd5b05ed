// Geometry of the quantisation work items (one 128x128 tile, or up to 128 consecutive 1x128
// blocks, per 512-lane workgroup) shared by the kernels that walk them.
#pragma once
#include "device_util.h"

namespace rs {

constexpr float kE4M3Max = 448.0f;

// -------------------------------------------------------------------------------------------
// block_quant work-item geometry.
// A workgroup of 512 lanes owns 128 "row slots" of up to 128 elements: the 128 rows of one
// 128x128 tile, or 128 consecutive 1x128 blocks.  Lane (r_in, cg) = (tid / 16, tid % 16) handles
// elements [8*cg, 8*cg + 8) of slots r_in + 32*i, i = 0..3, so one access instruction covers 32
// slots of 256 contiguous bytes each and a lane keeps four 16-byte vectors in flight.
// -------------------------------------------------------------------------------------------
constexpr int kQuantThreads = 512;
constexpr int kQuantLoads = kItemSlots * 16 / kQuantThreads;  // 4
constexpr int kQuantRowStep = kQuantThreads / 16;             // 32
static_assert(kQuantLoads == 4, "the lean path combines exactly four per-lane maxima");

struct Slot {
  int64_t off;   // element offset inside the tensor of this lane's 8 elements
  int64_t blk;   // scale index relative to the tensor (1x128 runs only)
  int ncol;      // how many of the 8 elements exist (0 = nothing to do)
};

__device__ __forceinline__ Slot tile_slot(const TensorDev& t, int64_t br, int bc, int slot, int col0) {
  Slot s;
  const int64_t row = br * 128 + slot;
  const int64_t col = int64_t(bc) * 128 + col0;
  s.off = row * t.cols + col;
  s.blk = 0;
  const int64_t left = t.cols - col;
  s.ncol = (row < t.rows && left > 0) ? int(min(int64_t(8), left)) : 0;
  return s;
}

__device__ __forceinline__ Slot run_slot(const TensorDev& t, int64_t b0, int count, int slot, int col0) {
  Slot s;
  s.blk = b0 + slot;
  s.off = 0;
  s.ncol = 0;
  if (slot >= count) return s;
  int64_t left;
  if (t.flags & kFlagContig) {
    s.off = s.blk * 128 + col0;
    left = t.e - s.off;
  } else {
    const int64_t r = s.blk / t.nbc;
    const int64_t col = (s.blk - r * t.nbc) * 128 + col0;
    s.off = r * t.cols + col;
    left = t.cols - col;
  }
  s.ncol = left > 0 ? int(min(int64_t(8), left)) : 0;
  return s;
}

__device__ __forceinline__ void zero_fill_bytes(uint8_t* dst, int count, int nthreads) {
  // dst need not be aligned: bytes up to the first 16-byte line, vectors, bytes after
  const int head = min(count, int((16 - (reinterpret_cast<uintptr_t>(dst) & 15)) & 15));
  const int nvec = (count - head) >> 4;
  const int tail = (count - head) & 15;
  const int tid = threadIdx.x;
  if (tid < head) dst[tid] = 0;
  for (int v = tid; v < nvec; v += nthreads) st16(dst + head + (v << 4), u32x4{0, 0, 0, 0});
  if (tid < tail) dst[head + (nvec << 4) + tid] = 0;
}

}  // namespace rs
