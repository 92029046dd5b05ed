// The fixed summation order of shard_reduce, shared by every kernel that forms the mean of W
// partials so that all of them give the same bits: partial w is added, in increasing w, to
// running sum w mod 8 (all eight start at +0); the eight sums combine pairwise,
// ((a0 + a1) + (a2 + a3)) + ((a4 + a5) + (a6 + a7)).  The factor 1/W is applied by the caller.
#pragma once
#include "device_util.h"

namespace rs {

__device__ __forceinline__ void add_bf16x8(float (&acc)[8], const u32x4 v) {
  acc[0] += __uint_as_float(v.x << 16);
  acc[1] += __uint_as_float(v.x & 0xffff0000u);
  acc[2] += __uint_as_float(v.y << 16);
  acc[3] += __uint_as_float(v.y & 0xffff0000u);
  acc[4] += __uint_as_float(v.z << 16);
  acc[5] += __uint_as_float(v.z & 0xffff0000u);
  acc[6] += __uint_as_float(v.w << 16);
  acc[7] += __uint_as_float(v.w & 0xffff0000u);
}

// 8 bf16 elements at p: one 16-byte vector, or (kVec false) the first ncol of them one by one,
// the rest reading as +0
template <bool kVec>
__device__ __forceinline__ u32x4 load_bf16x8(const uint16_t* p, int ncol) {
  if (kVec) return ld16(p);
  unsigned w[4] = {0, 0, 0, 0};
#pragma unroll
  for (int q = 0; q < 8; ++q)
    if (q < ncol) w[q >> 1] |= unsigned(p[q]) << ((q & 1) * 16);
  return u32x4{w[0], w[1], w[2], w[3]};
}

// rows w .. w + 7 of this lane's column; rows at or past W read as +0 (they keep the row -> set rule)
template <bool kVec>
__device__ __forceinline__ void load_rows(u32x4 (&v)[8], const uint16_t* p, int64_t row_stride, int w,
                                          int W, int ncol) {
  if (w + 8 <= W) {
#pragma unroll
    for (int a = 0; a < 8; ++a) v[a] = load_bf16x8<kVec>(p + int64_t(w + a) * row_stride, ncol);
  } else {
#pragma unroll
    for (int a = 0; a < 8; ++a)
      v[a] = w + a < W ? load_bf16x8<kVec>(p + int64_t(w + a) * row_stride, ncol) : u32x4{0, 0, 0, 0};
  }
}

// sum[q] = the ordered sum over the W rows of element q of the 8-element column at p (rows
// row_stride elements apart).  kDouble keeps the next eight rows in flight while the current
// ones are added.
template <bool kDouble, bool kVec>
__device__ __forceinline__ void reduce_column(const uint16_t* p, int64_t row_stride, int W, int ncol,
                                              float (&sum)[8]) {
  u32x4 v[8];
  load_rows<kVec>(v, p, row_stride, 0, W, ncol);
  float acc[8][8];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[a][q] = 0.0f;

  for (int w = 8;; w += 8) {   // v holds rows w - 8 .. w - 1
    if (kDouble) {
      u32x4 next[8];
      if (w < W) load_rows<kVec>(next, p, row_stride, w, W, ncol);
#pragma unroll
      for (int a = 0; a < 8; ++a) add_bf16x8(acc[a], v[a]);
      if (w >= W) break;
#pragma unroll
      for (int a = 0; a < 8; ++a) v[a] = next[a];
    } else {
#pragma unroll
      for (int a = 0; a < 8; ++a) add_bf16x8(acc[a], v[a]);
      if (w >= W) break;
      load_rows<kVec>(v, p, row_stride, w, W, ncol);
    }
  }
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const float s01 = acc[0][q] + acc[1][q], s23 = acc[2][q] + acc[3][q];
    const float s45 = acc[4][q] + acc[5][q], s67 = acc[6][q] + acc[7][q];
    sum[q] = (s01 + s23) + (s45 + s67);
  }
}

}  // namespace rs
