// HIP kernels for gfx950 (CDNA4, wave64): the four HBM-bound movers of the DBuffer hot path.
//
// Common shape: one 16-byte vector per lane per access and a very large grid (a plain copy on
// MI355X is fastest that way: no grid-stride loop, no multi-vector tiles), single-wavefront
// workgroups for the pure streaming kernels (measured 3-4 % faster than 256 lanes),
// non-temporal loads/stores since nothing is reused, and one scalar table lookup per
// workgroup to find its tensor.  No MFMA: nothing here is a contraction.
#include <hip/hip_runtime.h>

#include "rs_internal.h"
#include "rs_launch.h"

namespace rs {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

constexpr int kThreads = 256;
constexpr float kE4M3Max = 448.0f;

__device__ __forceinline__ u32x4 ld16(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
}
__device__ __forceinline__ void st16(void* p, u32x4 v) {
  __builtin_nontemporal_store(v, reinterpret_cast<u32x4*>(p));
}
__device__ __forceinline__ u32x2 ld8(const void* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
}
__device__ __forceinline__ void st8(void* p, u32x2 v) {
  __builtin_nontemporal_store(v, reinterpret_cast<u32x2*>(p));
}

// Workgroups are handed to the 8 XCDs round-robin by block index.  This turns the block index
// into a work index such that each XCD takes runs of `chunk` consecutive work items (work that is
// adjacent in memory then shares an XCD's L2 and DRAM pages).  The grid must be a multiple of
// 8 * chunk; indices at or past the real count are skipped by the caller.
constexpr int kXcdChunk = 16;  // measured best of 4..256 for block_quant and shard_reduce

__device__ __forceinline__ int64_t xcd_chunked(int64_t block, int chunk) {
  const int64_t x = block % 8, q = block / 8;
  return ((q / chunk) * 8 + x) * chunk + q % chunk;
}

// grid size for `count` work items under xcd_chunked(.., kXcdChunk)
static inline int64_t xcd_grid(int64_t count) {
  const int64_t unit = 8 * kXcdChunk;
  return (count + unit - 1) / unit * unit;
}

// -------------------------------------------------------------------------------------------
// Group-level operators of the DBuffer: one launch for all tensors of the unit.
//   pack (copy + zero), its inverse, pack with a scale factor, accumulate (axpy), scale.
// Four single-wavefront workgroups per granule (kGranule buffer elements of one rank region)
// that holds payload; the two pack forms add one workgroup per pure-padding granule to zero it,
// the others never touch padding.  fp32 arithmetic, one rounding to bf16 (nearest even).
// -------------------------------------------------------------------------------------------
constexpr int kCopyThreads = 64;
constexpr int kCopyParts = kGranule / (kCopyThreads * 8);  // workgroups per granule: 4

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// two fp32 -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  return __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}
__device__ __forceinline__ float bf16_lo(unsigned packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(unsigned packed) { return __uint_as_float(packed & 0xffff0000u); }

// d = bf16(d * alpha) / d = bf16(d + alpha * s) on a packed pair; separate multiply and add
__device__ __forceinline__ unsigned scale_pair(unsigned d, float alpha) {
  return pack_bf16(bf16_lo(d) * alpha, bf16_hi(d) * alpha);
}
__device__ __forceinline__ unsigned axpy_pair(unsigned d, unsigned s, float alpha) {
  const float lo = alpha * bf16_lo(s), hi = alpha * bf16_hi(s);
  return pack_bf16(bf16_lo(d) + lo, bf16_hi(d) + hi);
}
__device__ __forceinline__ u32x4 scale8(u32x4 d, float alpha) {
  return u32x4{scale_pair(d.x, alpha), scale_pair(d.y, alpha), scale_pair(d.z, alpha),
               scale_pair(d.w, alpha)};
}
__device__ __forceinline__ u32x4 axpy8(u32x4 d, u32x4 s, float alpha) {
  return u32x4{axpy_pair(d.x, s.x, alpha), axpy_pair(d.y, s.y, alpha), axpy_pair(d.z, s.z, alpha),
               axpy_pair(d.w, s.w, alpha)};
}

template <int kOp>
__global__ __launch_bounds__(kCopyThreads) void group_op_kernel(
    const TensorDev* __restrict__ T, int n, const int32_t* __restrict__ gran_first,
    const int32_t* __restrict__ granules, const int32_t* __restrict__ padding,
    unsigned n_copy_groups, void* const* __restrict__ ptrs, uint16_t* __restrict__ dbuf, int64_t S,
    int64_t gpr, float alpha) {
  constexpr bool kFillsPadding = kOp == kGroupPack || kOp == kGroupPackScaled;
  constexpr bool kReadsBuffer = kOp == kGroupUnpack || kOp == kGroupAdd || kOp == kGroupScale;
  constexpr bool kUsesTensors = kOp != kGroupScale;
  if (kFillsPadding && blockIdx.x >= n_copy_groups) {
    // a granule of nothing but padding: this wavefront zeroes all of it
    const int64_t gid = padding[blockIdx.x - n_copy_groups];
    const int64_t k = gid / gpr;
    const int64_t i0 = (gid - k * gpr) * kGranule;
    const int len = int(min(int64_t(kGranule), S - i0));
#pragma unroll
    for (int h = 0; h < kCopyParts; ++h) {
      const int lo = (h * kCopyThreads + int(threadIdx.x)) * 8;
      if (lo < len) st16(dbuf + k * S + i0 + lo, u32x4{0, 0, 0, 0});
    }
    return;
  }
  const unsigned slot = blockIdx.x / kCopyParts, part = blockIdx.x % kCopyParts;
  const int64_t bid = granules[slot];
  const int64_t k = bid / gpr;
  const int64_t i0 = (bid - k * gpr) * kGranule;
  const int64_t d0 = k * S + i0;
  const int len = int(min(int64_t(kGranule), S - i0));
  const int lane_off = (int(part) * kCopyThreads + int(threadIdx.x)) * 8;
  if (lane_off >= len) return;
  const int64_t d = d0 + lane_off;
  const int t0 = gran_first[bid];

  bool empty = t0 >= n;
  if (!empty) {
    const int64_t ell = T[t0].ell, end = ell + T[t0].e;
    if (ell <= d0 && d0 + len <= end) {
      // the whole granule lies inside tensor t0 (the common case by far)
      if (!kUsesTensors) {
        st16(dbuf + d, scale8(ld16(dbuf + d), alpha));
        return;
      }
      uint16_t* base = reinterpret_cast<uint16_t*>(ptrs[t0]) + (d0 - ell);
      if ((reinterpret_cast<uintptr_t>(base) & 15) == 0) {
        if (kOp == kGroupUnpack)
          st16(base + lane_off, ld16(dbuf + d));
        else if (kOp == kGroupPack)
          st16(dbuf + d, ld16(base + lane_off));
        else if (kOp == kGroupPackScaled)
          st16(dbuf + d, scale8(ld16(base + lane_off), alpha));
        else
          st16(dbuf + d, axpy8(ld16(dbuf + d), ld16(base + lane_off), alpha));
        return;
      }
    }
    empty = ell >= d0 + len;
  }
  if (empty) {  // nothing but padding here
    if (kFillsPadding) st16(dbuf + d, u32x4{0, 0, 0, 0});
    return;
  }

  // Mixed granule (tensor boundaries, padding, or a source that is not 16-byte aligned):
  // resolve every element on its own.
  int s = t0;
  uint16_t vals[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (kReadsBuffer) {
    const u32x4 v = ld16(dbuf + d);
    vals[0] = uint16_t(v.x); vals[1] = uint16_t(v.x >> 16);
    vals[2] = uint16_t(v.y); vals[3] = uint16_t(v.y >> 16);
    vals[4] = uint16_t(v.z); vals[5] = uint16_t(v.z >> 16);
    vals[6] = uint16_t(v.w); vals[7] = uint16_t(v.w >> 16);
  }
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const int64_t pos = d + q;
    while (s < n && T[s].ell + T[s].e <= pos) ++s;
    const bool inside = s < n && T[s].ell <= pos;
    if (!inside) continue;   // padding keeps what it holds (+0 for the pack forms)
    if (kOp == kGroupScale) {
      vals[q] = uint16_t(scale_pair(vals[q], alpha));
      continue;
    }
    uint16_t* elem = reinterpret_cast<uint16_t*>(ptrs[s]) + (pos - T[s].ell);
    if (kOp == kGroupUnpack)
      *elem = vals[q];
    else if (kOp == kGroupPack)
      vals[q] = *elem;
    else if (kOp == kGroupPackScaled)
      vals[q] = uint16_t(scale_pair(*elem, alpha));
    else
      vals[q] = uint16_t(axpy_pair(vals[q], *elem, alpha));
  }
  if (kOp != kGroupUnpack) {
    u32x4 v;
    v.x = vals[0] | (uint32_t(vals[1]) << 16);
    v.y = vals[2] | (uint32_t(vals[3]) << 16);
    v.z = vals[4] | (uint32_t(vals[5]) << 16);
    v.w = vals[6] | (uint32_t(vals[7]) << 16);
    st16(dbuf + d, v);
  }
}

// Pure writes want 256-lane workgroups with one vector per lane (measured 6.9 TB/s against
// 4.8 TB/s for single-wavefront workgroups and 6.4 TB/s for 4 vectors per lane), the opposite
// of what copies want.
constexpr int kFillThreads = 256;

// every element of a buffer of nvec 16-byte vectors becomes +0
__global__ __launch_bounds__(kFillThreads) void fill_zero_kernel(u32x4* __restrict__ dst, int64_t nvec) {
  const int64_t i = int64_t(blockIdx.x) * kFillThreads + threadIdx.x;
  if (i < nvec) dst[i] = u32x4{0, 0, 0, 0};
}

// -------------------------------------------------------------------------------------------
// shard_reduce: out[i] = (1/W) * sum_w P[w][i] on the payload of one rank region, 0 on padding.
// Each lane owns 8 consecutive elements and walks the W rows; rows are spread over 8
// accumulator sets (row w -> set w mod 8) that are combined pairwise at the end, so the
// summation order is fixed and the rounding error grows with W/8 + 3, not W.
// -------------------------------------------------------------------------------------------
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

// rows w .. w + 7 of this lane's column; rows at or past W read as +0 (they keep the row -> set rule)
__device__ __forceinline__ void load_rows(u32x4 (&v)[8], const uint16_t* p, int64_t row_stride, int w,
                                          int W) {
  if (w + 8 <= W) {
#pragma unroll
    for (int a = 0; a < 8; ++a) v[a] = ld16(p + int64_t(w + a) * row_stride);
  } else {
#pragma unroll
    for (int a = 0; a < 8; ++a)
      v[a] = w + a < W ? ld16(p + int64_t(w + a) * row_stride) : u32x4{0, 0, 0, 0};
  }
}

// kReduceThreads = 256: one granule per workgroup; 512: two granules (8 KiB contiguous per row).
// kDouble keeps the next eight rows in flight while the current ones are added.  Measured on
// regions of 4096 granules and more: 512 lanes with kDouble is the fastest shape (+5 % at
// W = 32, +3 % at W = 128); on short regions 256 lanes without it.  Requesting the first rows
// before the table lookups was tried and lost everywhere: what it reads on padding costs more
// than the latency it hides.
template <int kReduceThreads, bool kDouble>
__global__ __launch_bounds__(kReduceThreads) void shard_reduce_kernel(
    const TensorDev* __restrict__ T, int n, const int32_t* __restrict__ gran_first,
    const uint16_t* __restrict__ P, int64_t row_stride, float* __restrict__ out, int64_t S,
    int64_t gpr, int rank, int W, float inv_w) {
  // with 512 lanes, waves 0-3 take the even granule of the pair, waves 4-7 the odd one
  const int half = __builtin_amdgcn_readfirstlane(int(threadIdx.x) / kThreads);  // wave-uniform
  const int64_t j = xcd_chunked(blockIdx.x, kXcdChunk) * (kReduceThreads / kThreads) + half;
  if (j >= gpr) return;
  const int64_t i0 = j * kGranule;
  const int64_t d0 = int64_t(rank) * S + i0;
  const int len = int(min(int64_t(kGranule), S - i0));
  const int lane_off = (threadIdx.x % kThreads) * 8;
  if (lane_off >= len) return;
  const int64_t d = d0 + lane_off;
  float* o = out + i0 + lane_off;

  // payload mask of this lane's 8 elements
  const int t0 = gran_first[int64_t(rank) * gpr + j];
  unsigned mask = 0xffu;
  bool empty = t0 >= n;
  if (!empty) {
    const int64_t ell = T[t0].ell, end = ell + T[t0].e;
    empty = ell >= d0 + len;
    if (!empty && !(ell <= d0 && d0 + len <= end)) {
      mask = 0;
      int s = t0;
#pragma unroll
      for (int q = 0; q < 8; ++q) {
        const int64_t pos = d + q;
        while (s < n && T[s].ell + T[s].e <= pos) ++s;
        if (s < n && T[s].ell <= pos) mask |= 1u << q;
      }
    }
  }
  if (empty || mask == 0) {  // padding only: no reads at all
    st16(o, u32x4{0, 0, 0, 0});
    st16(o + 4, u32x4{0, 0, 0, 0});
    return;
  }

  const uint16_t* p = P + i0 + lane_off;
  u32x4 v[8];
  load_rows(v, p, row_stride, 0, W);
  float acc[8][8];
#pragma unroll
  for (int a = 0; a < 8; ++a)
#pragma unroll
    for (int q = 0; q < 8; ++q) acc[a][q] = 0.0f;

  for (int w = 8;; w += 8) {   // v holds rows w - 8 .. w - 1
    if (kDouble) {
      u32x4 next[8];
      if (w < W) load_rows(next, p, row_stride, w, W);
#pragma unroll
      for (int a = 0; a < 8; ++a) add_bf16x8(acc[a], v[a]);
      if (w >= W) break;
#pragma unroll
      for (int a = 0; a < 8; ++a) v[a] = next[a];
    } else {
#pragma unroll
      for (int a = 0; a < 8; ++a) add_bf16x8(acc[a], v[a]);
      if (w >= W) break;
      load_rows(v, p, row_stride, w, W);
    }
  }
  float r[8];
#pragma unroll
  for (int q = 0; q < 8; ++q) {
    const float s01 = acc[0][q] + acc[1][q], s23 = acc[2][q] + acc[3][q];
    const float s45 = acc[4][q] + acc[5][q], s67 = acc[6][q] + acc[7][q];
    const float m = ((s01 + s23) + (s45 + s67)) * inv_w;
    r[q] = (mask >> q) & 1u ? m : 0.0f;
  }
  st16(o, u32x4{__float_as_uint(r[0]), __float_as_uint(r[1]), __float_as_uint(r[2]),
                __float_as_uint(r[3])});
  st16(o + 4, u32x4{__float_as_uint(r[4]), __float_as_uint(r[5]), __float_as_uint(r[6]),
                    __float_as_uint(r[7])});
}

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

__device__ __forceinline__ unsigned abs_max_bits(unsigned m, unsigned packed) {
  // bf16 magnitudes order like their 15-bit patterns
  m = max(m, packed & 0x7fffu);
  return max(m, (packed >> 16) & 0x7fffu);
}

// The divisor of a block (its scale) is shared by all its elements, so the correctly rounded
// quotient x / scale is obtained without a per-element IEEE division sequence:
//   r  = RN(1 / b)                      one true division per block
//   q0 = RN(a * r)                      within 1.5 ulp of a / b
//   q1 = RN(q0 + RN(a - b * q0) * r)    a faithful rounding of a / b
//   q2 = RN(q1 + (a - b * q1) * r)      = RN(a / b): from a faithful q1 the residual is exact
//                                         in an FMA and this last step rounds correctly (Markstein)
// This holds while no intermediate under- or overflows, which kDivFastLo <= amax < kDivFastHi
// guarantees for every element whose quotient is not far below the smallest E4M3 subnormal
// (those give a zero code either way); blocks outside that range take the plain division.
// The sign is re-applied at the end because the corrections turn -0 into +0.
constexpr unsigned kDivFastLo = 67u << 7;    // amax >= 2^-60 (bf16 bit pattern)
constexpr unsigned kDivFastHi = 188u << 7;   // amax <  2^61

struct Divisor {
  float b, r;
  bool fast;
};

__device__ __forceinline__ Divisor make_divisor(unsigned amax_bits) {
  Divisor d;
  d.b = __uint_as_float(amax_bits << 16) / kE4M3Max;
  d.fast = amax_bits >= kDivFastLo && amax_bits < kDivFastHi;
  d.r = d.fast ? 1.0f / d.b : 0.0f;
  return d;
}

__device__ __forceinline__ float divide(float a, const Divisor& d) {
  if (!d.fast) return a / d.b;
  float q = a * d.r;
  float e = __builtin_fmaf(-q, d.b, a);
  q = __builtin_fmaf(e, d.r, q);
  e = __builtin_fmaf(-q, d.b, a);
  q = __builtin_fmaf(e, d.r, q);
  return __builtin_copysignf(q, a);
}

__device__ __forceinline__ unsigned quant_pair(unsigned packed, const Divisor& d) {
  // two bf16 -> two E4M3 codes in the low 16 bits
  const float a = divide(__uint_as_float(packed << 16), d);
  const float b = divide(__uint_as_float(packed & 0xffff0000u), d);
  const float ca = __builtin_amdgcn_fmed3f(a, -kE4M3Max, kE4M3Max);
  const float cb = __builtin_amdgcn_fmed3f(b, -kE4M3Max, kE4M3Max);
  return unsigned(__builtin_amdgcn_cvt_pk_fp8_f32(ca, cb, 0, false)) & 0xffffu;
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

// One full work item whose rows are 16-byte structured: 128 slots of exactly 128 elements,
// slot s at x + s * pitch.  kTile: one scale for the whole item (a 128x128 tile);
// otherwise one scale per slot (128 consecutive 1x128 blocks), written to scales[slot].
template <bool kTile>
__device__ __forceinline__ void quant_full_item(const uint16_t* __restrict__ x,
                                                uint8_t* __restrict__ codes, int64_t pitch,
                                                float* __restrict__ scales, unsigned* wave_max) {
  const int tid = threadIdx.x;
  const int64_t lane_off = int64_t(tid >> 4) * pitch + (tid & 15) * 8;
  const int64_t step = int64_t(kQuantRowStep) * pitch;
  u32x4 v[kQuantLoads];
#pragma unroll
  for (int i = 0; i < kQuantLoads; ++i) v[i] = ld16(x + lane_off + i * step);
  unsigned m[kQuantLoads];
#pragma unroll
  for (int i = 0; i < kQuantLoads; ++i) {
    unsigned a = abs_max_bits(0, v[i].x);
    a = abs_max_bits(a, v[i].y);
    a = abs_max_bits(a, v[i].z);
    m[i] = abs_max_bits(a, v[i].w);
  }
  if (kTile) {
    unsigned a = max(max(m[0], m[1]), max(m[2], m[3]));
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) a = max(a, unsigned(__shfl_xor(int(a), off)));
    if ((tid & 63) == 0) wave_max[tid >> 6] = a;
    __syncthreads();
    a = wave_max[0];
#pragma unroll
    for (int w = 1; w < kQuantThreads / 64; ++w) a = max(a, wave_max[w]);
    if (tid == 0) scales[0] = __uint_as_float(a << 16) / kE4M3Max;
#pragma unroll
    for (int i = 0; i < kQuantLoads; ++i) m[i] = a;
  } else {
#pragma unroll
    for (int i = 0; i < kQuantLoads; ++i) {
      unsigned a = m[i];
#pragma unroll
      for (int off = 8; off >= 1; off >>= 1) a = max(a, unsigned(__shfl_xor(int(a), off)));
      m[i] = a;
      if ((tid & 15) == 0) scales[(tid >> 4) + kQuantRowStep * i] = __uint_as_float(a << 16) / kE4M3Max;
    }
  }
#pragma unroll
  for (int i = 0; i < kQuantLoads; ++i) {
    u32x2 c{0, 0};
    if (m[i] != 0) {
      const Divisor d = make_divisor(m[i]);
      c.x = quant_pair(v[i].x, d) | (quant_pair(v[i].y, d) << 16);
      c.y = quant_pair(v[i].z, d) | (quant_pair(v[i].w, d) << 16);
    }
    st8(codes + lane_off + i * step, c);
  }
}

// -------------------------------------------------------------------------------------------
// block_quant: amax per block (wavefront shuffles, LDS across the 8 waves of a tile),
// scale = amax / 448, codes = E4M3(clamp(x / scale)) with the hardware RNE convert.
// x / codes are addressed relative to elem_base (0 or rank * S), scales to scale_off.
// -------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kQuantThreads) void block_quant_kernel(
    const TensorDev* __restrict__ T, const Item* __restrict__ items, int64_t item_off,
    const uint16_t* __restrict__ x_one, uint8_t* __restrict__ codes_one,
    float* __restrict__ scales_one, void* const* __restrict__ batch, int batch_count,
    int64_t elem_base, int64_t scale_off, int64_t item_count) {
  __shared__ unsigned wave_max[kQuantThreads / 64];
  // batched launch: batch = [shards | codes | scales] pointers of batch_count units
  const uint16_t* __restrict__ x = x_one;
  uint8_t* __restrict__ codes = codes_one;
  float* __restrict__ scales = scales_one;
  // adjacent tiles of a row of tiles share DRAM pages and cache lines: keep them on one XCD
  int64_t idx = xcd_chunked(blockIdx.x, kXcdChunk);
  if (batch) {
    // the units' item ranges are laid end to end in one flat grid: no idle tail per unit
    const int64_t u = idx / item_count;
    if (u >= batch_count) return;
    idx -= u * item_count;
    x = static_cast<const uint16_t*>(batch[u]);
    codes = static_cast<uint8_t*>(batch[batch_count + u]);
    scales = static_cast<float*>(batch[2 * batch_count + u]);
  } else if (idx >= item_count) {
    return;
  }
  const Item it = items[item_off + idx];
  if (it.tensor < 0) {
    zero_fill_bytes(codes + (it.first - elem_base), it.count, kQuantThreads);
    return;
  }
  const TensorDev t = T[it.tensor];
  const bool tile = (t.flags & kFlagTile) != 0;
  const bool vec = (t.flags & kFlagVec) != 0;
  const int tid = threadIdx.x;
  const int r_in = tid >> 4, col0 = (tid & 15) * 8;
  const int64_t base = t.ell - elem_base;

  // Full, 16-byte-structured items (nearly all of them) take the lean path: no per-slot
  // bookkeeping, straight-line loads, one reduction, straight-line stores.
  if (vec) {
    if (tile) {
      if ((it.first + 1) * 128 <= t.rows && int64_t(it.count + 1) * 128 <= t.cols) {
        const int64_t off = base + it.first * 128 * t.cols + int64_t(it.count) * 128;
        quant_full_item<true>(x + off, codes + off, t.cols,
                              scales + (t.scale_base + it.first * t.nbc + it.count - scale_off),
                              wave_max);
        return;
      }
    } else if ((t.flags & kFlagContig) && it.count == kItemSlots &&
               (it.first + kItemSlots) * 128 <= t.e) {
      const int64_t off = base + it.first * 128;
      quant_full_item<false>(x + off, codes + off, 128,
                             scales + (t.scale_base + it.first - scale_off), wave_max);
      return;
    }
  }

  Slot sl[kQuantLoads];
  u32x4 v[kQuantLoads];
#pragma unroll
  for (int i = 0; i < kQuantLoads; ++i) {
    sl[i] = tile ? tile_slot(t, it.first, it.count, r_in + kQuantRowStep * i, col0)
                 : run_slot(t, it.first, it.count, r_in + kQuantRowStep * i, col0);
    v[i] = u32x4{0, 0, 0, 0};
    if (sl[i].ncol == 0) continue;
    const uint16_t* src = x + base + sl[i].off;
    if (vec) {
      v[i] = ld16(src);
      if (sl[i].ncol < 8) {  // drop what belongs to the next row / lies past the tensor
        unsigned w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
        for (int q = 0; q < 8; ++q)
          if (q >= sl[i].ncol) w[q >> 1] &= (q & 1) ? 0x0000ffffu : 0xffff0000u;
        v[i] = u32x4{w[0], w[1], w[2], w[3]};
      }
    } else {
      unsigned w[4] = {0, 0, 0, 0};
#pragma unroll
      for (int q = 0; q < 8; ++q)
        if (q < sl[i].ncol) w[q >> 1] |= unsigned(src[q]) << ((q & 1) * 16);
      v[i] = u32x4{w[0], w[1], w[2], w[3]};
    }
  }

  // per-slot amax over this lane's 8 elements, then over the 16 lanes of the slot
  unsigned m[kQuantLoads];
#pragma unroll
  for (int i = 0; i < kQuantLoads; ++i) {
    unsigned a = 0;
    a = abs_max_bits(a, v[i].x);
    a = abs_max_bits(a, v[i].y);
    a = abs_max_bits(a, v[i].z);
    a = abs_max_bits(a, v[i].w);
    m[i] = a;
  }
  if (tile) {
    unsigned a = m[0];
#pragma unroll
    for (int i = 1; i < kQuantLoads; ++i) a = max(a, m[i]);
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) a = max(a, unsigned(__shfl_xor(int(a), off)));
    if ((tid & 63) == 0) wave_max[tid >> 6] = a;
    __syncthreads();
    a = wave_max[0];
#pragma unroll
    for (int w = 1; w < kQuantThreads / 64; ++w) a = max(a, wave_max[w]);
#pragma unroll
    for (int i = 0; i < kQuantLoads; ++i) m[i] = a;
    if (tid == 0) {
      const int64_t sidx = t.scale_base + it.first * t.nbc + it.count - scale_off;
      scales[sidx] = __uint_as_float(a << 16) / kE4M3Max;
    }
  } else {
#pragma unroll
    for (int i = 0; i < kQuantLoads; ++i) {
      unsigned a = m[i];
#pragma unroll
      for (int off = 8; off >= 1; off >>= 1) a = max(a, unsigned(__shfl_xor(int(a), off)));
      m[i] = a;
      if ((tid & 15) == 0 && r_in + kQuantRowStep * i < it.count)
        scales[t.scale_base + sl[i].blk - scale_off] = __uint_as_float(a << 16) / kE4M3Max;
    }
  }

#pragma unroll
  for (int i = 0; i < kQuantLoads; ++i) {
    if (sl[i].ncol == 0) continue;
    u32x2 c{0, 0};
    if (m[i] != 0) {
      const Divisor d = make_divisor(m[i]);
      c.x = quant_pair(v[i].x, d) | (quant_pair(v[i].y, d) << 16);
      c.y = quant_pair(v[i].z, d) | (quant_pair(v[i].w, d) << 16);
    }
    uint8_t* dst = codes + base + sl[i].off;
    if (vec && sl[i].ncol == 8) {
      st8(dst, c);
    } else {
#pragma unroll
      for (int q = 0; q < 8; ++q)
        if (q < sl[i].ncol) dst[q] = uint8_t((q < 4 ? c.x : c.y) >> ((q & 3) * 8));
    }
  }
}

// -------------------------------------------------------------------------------------------
// dequant_unpack: codes of the gathered unit -> per-tensor bf16, value(code) * scale then RNE.
// Buffer-driven like ragged_pack: one single-wavefront workgroup per granule that holds
// payload; a lane converts 8 codes (one 8-byte load, one 16-byte store) in each quarter of the
// granule.  No block-wide step is needed, only the block's scale.
// -------------------------------------------------------------------------------------------
__device__ __forceinline__ unsigned bf16_rne(float f) {
  const unsigned u = __float_as_uint(f);
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

__device__ __forceinline__ void dequant4(unsigned word, float scale, unsigned& lo, unsigned& hi) {
  const auto a = __builtin_amdgcn_cvt_pk_f32_fp8(int(word), false);  // bytes 0, 1
  const auto b = __builtin_amdgcn_cvt_pk_f32_fp8(int(word), true);   // bytes 2, 3
  lo = pack_bf16(a[0] * scale, a[1] * scale);
  hi = pack_bf16(b[0] * scale, b[1] * scale);
}

// scale index (relative to the tensor) of the element at (row, col)
__device__ __forceinline__ int64_t scale_index(const TensorDev& t, int64_t row, int64_t col) {
  return ((t.flags & kFlagTile) ? (row >> 7) : row) * t.nbc + (col >> 7);
}

constexpr int kDequantThreads = 64;

// kF32: the tensors are fp32 (value * scale, no further rounding) instead of bf16
template <bool kF32>
__global__ __launch_bounds__(kDequantThreads) void dequant_unpack_kernel(
    const TensorDev* __restrict__ T, int n, const int32_t* __restrict__ gran_first,
    const int32_t* __restrict__ granules, const uint8_t* __restrict__ codes,
    const float* __restrict__ scales, void* const* __restrict__ ptrs, int64_t S, int64_t gpr) {
  const int64_t gid = granules[blockIdx.x];
  const int64_t k = gid / gpr;
  const int64_t i0 = (gid - k * gpr) * kGranule;
  const int64_t d0 = k * S + i0;
  const int len = int(min(int64_t(kGranule), S - i0));
  const int t0 = gran_first[gid];  // a payload granule: t0 < n
  // A lane converts kGroup codes per access so that its store is one 16-byte vector and a
  // wavefront's stores are contiguous: 8 codes -> 8 bf16, or 4 codes -> 4 fp32.
  constexpr int kGroup = kF32 ? 4 : 8;
  constexpr int kStep = kDequantThreads * kGroup;   // codes per access of the wavefront
  constexpr int kParts = kGranule / kStep;
  const int lane = threadIdx.x * kGroup;

  {
    const TensorDev t = T[t0];
    uint16_t* out = reinterpret_cast<uint16_t*>(ptrs[t0]);
    float* out32 = reinterpret_cast<float*>(ptrs[t0]);
    const bool inside = t.ell <= d0 && d0 + len <= t.ell + t.e;
    if (inside && (t.flags & kFlagVec) && (reinterpret_cast<uintptr_t>(out) & 15) == 0 &&
        t.cols < (int64_t(1) << 30)) {
      // The whole granule lies in one tensor whose rows keep every 8-element group inside one
      // row and one block.  (row, col) of the granule's first element once per workgroup
      // (exact: a double holds any element index below 2^53), then 32-bit steps per lane.
      const int64_t first = d0 - t.ell;
      int64_t row0 = int64_t(double(first) / double(t.cols));
      int64_t col0 = first - row0 * t.cols;
      if (col0 < 0) { col0 += t.cols; --row0; }
      if (col0 >= t.cols) { col0 -= t.cols; ++row0; }
      const unsigned C = unsigned(t.cols);
      const bool contig = (t.flags & kFlagContig) && !(t.flags & kFlagTile);
      u32x2 c[kParts];
      float sc[kParts];
      bool on[kParts];
#pragma unroll
      for (int h = 0; h < kParts; ++h) {
        const int lo = h * kStep + lane;
        on[h] = lo < len;
        if (!on[h]) continue;
        if (kF32)
          c[h] = u32x2{__builtin_nontemporal_load(reinterpret_cast<const unsigned*>(codes + d0 + lo)), 0};
        else
          c[h] = ld8(codes + d0 + lo);
        int64_t sidx;
        if (contig) {
          sidx = (first + lo) >> 7;            // blocks are consecutive runs of 128 elements
        } else {
          const unsigned cc = unsigned(col0) + unsigned(lo);
          const unsigned dr = cc / C;
          sidx = scale_index(t, row0 + dr, cc - dr * C);
        }
        sc[h] = scales[t.scale_base + sidx];
      }
#pragma unroll
      for (int h = 0; h < kParts; ++h) {
        if (!on[h]) continue;
        if (kF32) {
          const auto a = __builtin_amdgcn_cvt_pk_f32_fp8(int(c[h].x), false);
          const auto b = __builtin_amdgcn_cvt_pk_f32_fp8(int(c[h].x), true);
          st16(out32 + first + h * kStep + lane,
               u32x4{__float_as_uint(a[0] * sc[h]), __float_as_uint(a[1] * sc[h]),
                     __float_as_uint(b[0] * sc[h]), __float_as_uint(b[1] * sc[h])});
          continue;
        }
        unsigned o0, o1, o2, o3;
        dequant4(c[h].x, sc[h], o0, o1);
        dequant4(c[h].y, sc[h], o2, o3);
        st16(out + first + h * kStep + lane, u32x4{o0, o1, o2, o3});
      }
      return;
    }
  }

  // Granule with tensor boundaries or padding, or a tensor without 16-byte structure:
  // every element finds its tensor, row and column on its own.
  int s = t0;
  for (int h = 0; h < kParts; ++h) {
    const int lo = h * kStep + lane;
    if (lo >= len) break;
    for (int q = 0; q < kGroup; ++q) {
      const int64_t pos = d0 + lo + q;
      while (s < n && T[s].ell + T[s].e <= pos) ++s;
      if (s >= n || T[s].ell > pos) continue;
      const TensorDev t = T[s];
      const int64_t i = pos - t.ell;
      const int64_t row = i / t.cols;
      const int64_t col = i - row * t.cols;
      const float scale = scales[t.scale_base + scale_index(t, row, col)];
      const auto f = __builtin_amdgcn_cvt_pk_f32_fp8(int(codes[pos]), false);
      if (kF32)
        reinterpret_cast<float*>(ptrs[s])[i] = f[0] * scale;
      else
        reinterpret_cast<uint16_t*>(ptrs[s])[i] = uint16_t(bf16_rne(f[0] * scale));
    }
  }
}

// -------------------------------------------------------------------------------------------
// adam8_step: AdamW on the local shard with block-wise 8-bit moments.
// A workgroup of 1024 lanes owns one state work item: 32 rows x 256 columns of a 2-D tensor (a
// row of eight 32x32 state tiles), or 64 runs of 128 elements of a 1-D tensor seen as 32 rows of
// 256 elements.  Lane (cq, rw) = (tid % 64, tid / 64) handles the 4 elements at column 4 * cq of
// rows rw and rw + 16, so one access instruction of a wavefront covers one row (1 KiB of fp32)
// and a lane's two slots lie in one tile.  (Measured: 256 columns per item beat 512 and 1024,
// and beat one tile per wavefront by far - narrow row pieces waste DRAM pages; 1024 lanes beat
// 512 and 256.)  Items that are full and 16-byte structured skip all masking.  Pass 1 loads everything, applies the update,
// stores the master weight and the bf16 parameter and keeps the new moments in registers;
// after the block maxima are known (shuffles inside a wavefront, LDS across the
// wavefronts of a tile) pass 2 quantises and stores the codes.  One HBM read and one write
// per array.
// -------------------------------------------------------------------------------------------
constexpr int kStateThreads = 1024;
constexpr int kStateWaves = kStateThreads / 64;
constexpr int kStateSlots = 32 / kStateWaves;  // rows per lane

struct StateSlot {
  int64_t off;  // offset of the slot's first element in the rank's region
  int blk;      // state block, relative to the rank's first
  int nv;       // how many of the 4 elements exist (0: nothing to do)
};

template <bool kTile>
__device__ __forceinline__ StateSlot state_slot(const TensorDev& t, const Item& it, int row_in, int cq,
                                                int64_t base, int64_t state_off) {
  StateSlot s;
  s.off = 0;
  s.blk = 0;
  s.nv = 0;
  if (kTile) {
    const int64_t row = it.first * 32 + row_in;
    const int64_t col = int64_t(it.count) * kStateCols + 4 * cq;
    const int64_t left = t.cols - col;
    if (row < t.rows && left > 0) {
      s.nv = int(min(int64_t(4), left));
      s.off = base + row * t.cols + col;
      s.blk = int(t.state_base + it.first * t.sbc + (col >> 5) - state_off);
    }
  } else {
    const int run = 2 * row_in + (cq >> 5);
    const int64_t elem = (it.first + run) * 128 + 4 * (cq & 31);
    const int64_t left = t.e - elem;
    if (run < it.count && left > 0) {
      s.nv = int(min(int64_t(4), left));
      s.off = base + elem;
      s.blk = int(t.state_base + it.first + run - state_off);
    }
  }
  return s;
}

__device__ __forceinline__ float quant_step(float absmax, float levels) { return absmax / levels; }

// A divisor shared by many dividends, with the exact-division shortcut described at `divide`
// above.  It is taken while the divisor lies in [2^-60, 2^60]: every dividend used with it here
// is either at most a few hundred times the divisor in magnitude or a square root (never
// subnormal unless zero), so no intermediate of a quotient that matters under- or overflows.
__device__ __forceinline__ Divisor shared_divisor(float b) {
  Divisor d;
  d.b = b;
  const unsigned e = (__float_as_uint(b) >> 23) & 0xffu;
  d.fast = e >= 67u && e < 187u;
  d.r = d.fast ? 1.0f / b : 0.0f;
  return d;
}

// code = rint(x / step) clamped to [lo, hi]; an all-zero block (absmax 0) gives 0
__device__ __forceinline__ int state_code(float x, float absmax, const Divisor& step, float lo, float hi) {
  if (absmax == 0.0f) return 0;
  return int(__builtin_amdgcn_fmed3f(__builtin_rintf(divide(x, step)), lo, hi));
}

template <bool kTile, bool kFull>
__device__ __forceinline__ void adam8_item(const TensorDev& t, const Item& it,
                                           const float* __restrict__ g, float* __restrict__ w,
                                           uint16_t* __restrict__ p, uint8_t* __restrict__ mc,
                                           uint8_t* __restrict__ vc, float* __restrict__ am,
                                           float* __restrict__ av, int64_t elem_base,
                                           int64_t state_off, const Adam8Consts& c,
                                           float (*tile_max)[kStateThreads / 64][kStateCols / 32]) {
  const int tid = threadIdx.x;
  const int cq = tid & 63, rw = tid >> 6;
  const bool vec = kFull || (t.flags & kFlagVec4) != 0;
  const int64_t base = t.ell - elem_base;

  StateSlot sl[kStateSlots];
  u32x4 gv[kStateSlots], wv[kStateSlots];
  unsigned mcode[kStateSlots], vcode[kStateSlots];
#pragma unroll
  for (int i = 0; i < kStateSlots; ++i) {
    if (kFull) {  // a whole row of tiles inside the tensor: no masks
      const int64_t col = int64_t(it.count) * kStateCols + 4 * cq;
      sl[i].nv = 4;
      sl[i].off = base + (it.first * 32 + rw + kStateWaves * i) * t.cols + col;
      sl[i].blk = int(t.state_base + it.first * t.sbc + (col >> 5) - state_off);
    } else {
      sl[i] = state_slot<kTile>(t, it, rw + kStateWaves * i, cq, base, state_off);
    }
    gv[i] = wv[i] = u32x4{0, 0, 0, 0};
    mcode[i] = vcode[i] = 0;
    if (!kFull && sl[i].nv == 0) continue;
    if (kFull || (vec && sl[i].nv == 4)) {
      gv[i] = ld16(g + sl[i].off);
      wv[i] = ld16(w + sl[i].off);
      mcode[i] = __builtin_nontemporal_load(reinterpret_cast<const unsigned*>(mc + sl[i].off));
      vcode[i] = __builtin_nontemporal_load(reinterpret_cast<const unsigned*>(vc + sl[i].off));
    } else {
      unsigned gq[4] = {0, 0, 0, 0}, wq[4] = {0, 0, 0, 0};
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (j < sl[i].nv) {
          gq[j] = __float_as_uint(g[sl[i].off + j]);
          wq[j] = __float_as_uint(w[sl[i].off + j]);
          mcode[i] |= unsigned(mc[sl[i].off + j]) << (8 * j);
          vcode[i] |= unsigned(vc[sl[i].off + j]) << (8 * j);
        }
      gv[i] = u32x4{gq[0], gq[1], gq[2], gq[3]};
      wv[i] = u32x4{wq[0], wq[1], wq[2], wq[3]};
    }
  }

  // quantisation steps of the stored moments: one block per lane (tiles) or per slot (runs)
  float sm[kStateSlots], sv[kStateSlots];
  if (kTile) {
    float a = 0.0f, b = 0.0f;
    if (kFull || sl[0].nv > 0) {
      a = quant_step(am[sl[0].blk], 127.0f);
      b = quant_step(av[sl[0].blk], 255.0f);
    }
#pragma unroll
    for (int i = 0; i < kStateSlots; ++i) {
      sm[i] = a;
      sv[i] = b;
    }
  } else {
#pragma unroll
    for (int i = 0; i < kStateSlots; ++i) {
      sm[i] = sv[i] = 0.0f;
      if (sl[i].nv > 0) {
        sm[i] = quant_step(am[sl[i].blk], 127.0f);
        sv[i] = quant_step(av[sl[i].blk], 255.0f);
      }
    }
  }

  // pass 1: the update; new moments stay in registers
  const Divisor bc2 = shared_divisor(c.bc2_sqrt);
  float m[kStateSlots][4], v[kStateSlots][4];
  float mmax[kStateSlots], vmax[kStateSlots];
#pragma unroll
  for (int i = 0; i < kStateSlots; ++i) {
    const unsigned gq[4] = {gv[i].x, gv[i].y, gv[i].z, gv[i].w};
    const unsigned wq[4] = {wv[i].x, wv[i].y, wv[i].z, wv[i].w};
    float wn[4];
    mmax[i] = vmax[i] = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const float gj = __uint_as_float(gq[j]);
      const float m_old = float(int(int8_t(mcode[i] >> (8 * j)))) * sm[i];
      const float v_old = float((vcode[i] >> (8 * j)) & 0xffu) * sv[i];
      const float t1 = c.beta1 * m_old, t2 = c.one_minus_beta1 * gj;
      m[i][j] = t1 + t2;
      const float gg = gj * gj;
      const float t3 = c.beta2 * v_old, t4 = c.one_minus_beta2 * gg;
      v[i][j] = t3 + t4;
      const float w1 = __uint_as_float(wq[j]) * c.decay;
      const float root = divide(__builtin_sqrtf(v[i][j]), bc2);
      const float denom = root + c.eps;
      const float upd = c.step_size * (m[i][j] / denom);
      wn[j] = w1 - upd;
      mmax[i] = fmaxf(mmax[i], __builtin_fabsf(m[i][j]));
      vmax[i] = fmaxf(vmax[i], v[i][j]);
    }
    if (!kFull && sl[i].nv == 0) continue;
    if (kFull || (vec && sl[i].nv == 4)) {
      st16(w + sl[i].off, u32x4{__float_as_uint(wn[0]), __float_as_uint(wn[1]), __float_as_uint(wn[2]),
                                __float_as_uint(wn[3])});
      if (p) st8(p + sl[i].off, u32x2{pack_bf16(wn[0], wn[1]), pack_bf16(wn[2], wn[3])});
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (j < sl[i].nv) {
          w[sl[i].off + j] = wn[j];
          if (p) p[sl[i].off + j] = uint16_t(pack_bf16(wn[j], 0.0f));
        }
    }
  }

  // block maxima
  if (kTile) {
    float a = mmax[0], b = vmax[0];
#pragma unroll
    for (int i = 1; i < kStateSlots; ++i) {
      a = fmaxf(a, mmax[i]);
      b = fmaxf(b, vmax[i]);
    }
#pragma unroll
    for (int off = 1; off <= 4; off <<= 1) {
      a = fmaxf(a, __shfl_xor(a, off));
      b = fmaxf(b, __shfl_xor(b, off));
    }
    if ((cq & 7) == 0) {
      tile_max[0][rw][cq >> 3] = a;
      tile_max[1][rw][cq >> 3] = b;
    }
    __syncthreads();
    a = tile_max[0][0][cq >> 3];
    b = tile_max[1][0][cq >> 3];
#pragma unroll
    for (int q = 1; q < kStateThreads / 64; ++q) {
      a = fmaxf(a, tile_max[0][q][cq >> 3]);
      b = fmaxf(b, tile_max[1][q][cq >> 3]);
    }
    if (rw == 0 && (cq & 7) == 0 && (kFull || sl[0].nv > 0)) {
      am[sl[0].blk] = a;
      av[sl[0].blk] = b;
    }
#pragma unroll
    for (int i = 0; i < kStateSlots; ++i) {
      mmax[i] = a;
      vmax[i] = b;
    }
  } else {
#pragma unroll
    for (int i = 0; i < kStateSlots; ++i) {
      float a = mmax[i], b = vmax[i];
#pragma unroll
      for (int off = 1; off <= 16; off <<= 1) {
        a = fmaxf(a, __shfl_xor(a, off));
        b = fmaxf(b, __shfl_xor(b, off));
      }
      mmax[i] = a;
      vmax[i] = b;
      if ((cq & 31) == 0 && sl[i].nv > 0) {
        am[sl[i].blk] = a;
        av[sl[i].blk] = b;
      }
    }
  }

  // pass 2: quantise the new moments
#pragma unroll
  for (int i = 0; i < kStateSlots; ++i) {
    if (!kFull && sl[i].nv == 0) continue;
    const Divisor s1 = shared_divisor(quant_step(mmax[i], 127.0f));
    const Divisor s2 = shared_divisor(quant_step(vmax[i], 255.0f));
    unsigned cm = 0, cv = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      cm |= (unsigned(state_code(m[i][j], mmax[i], s1, -127.0f, 127.0f)) & 0xffu) << (8 * j);
      cv |= (unsigned(state_code(v[i][j], vmax[i], s2, 0.0f, 255.0f)) & 0xffu) << (8 * j);
    }
    if (kFull || (vec && sl[i].nv == 4)) {
      __builtin_nontemporal_store(cm, reinterpret_cast<unsigned*>(mc + sl[i].off));
      __builtin_nontemporal_store(cv, reinterpret_cast<unsigned*>(vc + sl[i].off));
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (j < sl[i].nv) {
          mc[sl[i].off + j] = uint8_t(cm >> (8 * j));
          vc[sl[i].off + j] = uint8_t(cv >> (8 * j));
        }
    }
  }
}

__global__ __launch_bounds__(kStateThreads) void adam8_step_kernel(
    const TensorDev* __restrict__ T, const Item* __restrict__ items, int64_t item_off,
    int64_t item_count, const float* __restrict__ g, float* __restrict__ w,
    uint16_t* __restrict__ p, uint8_t* __restrict__ mc, uint8_t* __restrict__ vc,
    float* __restrict__ am, float* __restrict__ av, void* const* __restrict__ batch,
    int batch_count, int64_t elem_base, int64_t state_off, Adam8Consts c) {
  __shared__ float tile_max[2][kStateThreads / 64][kStateCols / 32];
  // neighbouring column strips of a row of tiles share DRAM pages: keep them on one XCD
  int64_t idx = xcd_chunked(blockIdx.x, kXcdChunk);
  if (batch) {
    // the same shard of batch_count units, their item ranges end to end in one flat grid;
    // batch = [grad | master | param | m codes | v codes | m absmax | v absmax] pointers
    const int64_t u = idx / item_count;
    if (u >= batch_count) return;
    idx -= u * item_count;
    g = static_cast<const float*>(batch[u]);
    w = static_cast<float*>(batch[batch_count + u]);
    p = static_cast<uint16_t*>(batch[2 * batch_count + u]);
    mc = static_cast<uint8_t*>(batch[3 * batch_count + u]);
    vc = static_cast<uint8_t*>(batch[4 * batch_count + u]);
    am = static_cast<float*>(batch[5 * batch_count + u]);
    av = static_cast<float*>(batch[6 * batch_count + u]);
  } else if (idx >= item_count) {
    return;
  }
  const Item it = items[item_off + idx];
  const TensorDev t = T[it.tensor];
  if (t.flags & kFlagOneD)
    adam8_item<false, false>(t, it, g, w, p, mc, vc, am, av, elem_base, state_off, c, tile_max);
  else if ((t.flags & kFlagVec4) && (it.first + 1) * 32 <= t.rows &&
           int64_t(it.count + 1) * kStateCols <= t.cols)
    adam8_item<true, true>(t, it, g, w, p, mc, vc, am, av, elem_base, state_off, c, tile_max);
  else
    adam8_item<true, false>(t, it, g, w, p, mc, vc, am, av, elem_base, state_off, c, tile_max);
}

// -------------------------------------------------------------------------------------------
// plain copy: the measured ceiling and the counter calibration launch
// -------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kCopyThreads) void copy_probe_kernel(const u32x4* __restrict__ src,
                                                                 u32x4* __restrict__ dst,
                                                                 int64_t nvec) {
  const int64_t i = int64_t(blockIdx.x) * kCopyThreads + threadIdx.x;
  if (i < nvec) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// -------------------------------------------------------------------------------------------
// launchers (host)
// -------------------------------------------------------------------------------------------
static int launched() { return hipGetLastError() == hipSuccess ? RS_OK : RS_EHIP; }

int launch_group_op(int op, const DeviceTables& dev, int n, void* const* ptrs, void* dbuf, float alpha,
                    int64_t S, int64_t gpr, int64_t n_payload_gran, int64_t n_padding_gran,
                    hipStream_t st) {
  const bool fills = op == kGroupPack || op == kGroupPackScaled;
  uint16_t* db = static_cast<uint16_t*>(dbuf);
  const int64_t copy_groups = n_payload_gran * kCopyParts;
  // padding is zeroed by extra workgroups of the same launch (a separate fill launch was
  // measured slower even where padding is 88 % of the buffer)
  const int64_t grid = copy_groups + (fills ? n_padding_gran : 0);
  if (grid == 0) return RS_OK;
  if (grid < 0 || grid > 0x7fffffffLL) return RS_EOVERFLOW;
  const dim3 g{unsigned(grid)}, b{unsigned(kCopyThreads)};
#define RS_GROUP_OP(OP)                                                                         \
  group_op_kernel<OP><<<g, b, 0, st>>>(dev.tensors, n, dev.gran_first, dev.payload_gran,       \
                                       dev.padding_gran, unsigned(copy_groups), ptrs, db, S,   \
                                       gpr, alpha)
  switch (op) {
    case kGroupPack: RS_GROUP_OP(kGroupPack); break;
    case kGroupUnpack: RS_GROUP_OP(kGroupUnpack); break;
    case kGroupPackScaled: RS_GROUP_OP(kGroupPackScaled); break;
    case kGroupAdd: RS_GROUP_OP(kGroupAdd); break;
    case kGroupScale: RS_GROUP_OP(kGroupScale); break;
    default: return RS_EINVAL;
  }
#undef RS_GROUP_OP
  return launched();
}

int launch_fill_zero(void* dst, int64_t bytes, hipStream_t st) {
  const int64_t nvec = bytes / 16;
  const int64_t grid = (nvec + kFillThreads - 1) / kFillThreads;
  if (grid == 0) return RS_OK;
  if (grid > 0x7fffffffLL) return RS_EOVERFLOW;
  fill_zero_kernel<<<dim3(unsigned(grid)), dim3(kFillThreads), 0, st>>>(static_cast<u32x4*>(dst), nvec);
  return launched();
}

int launch_shard_reduce(const DeviceTables& dev, int n, const void* partials, int64_t row_stride,
                        float* out, int64_t S, int64_t gpr, int rank, int world, hipStream_t st) {
  if (gpr <= 0 || gpr > 0x7fffffffLL) return RS_EOVERFLOW;
  const float inv_w = 1.0f / float(world);
  const uint16_t* P = static_cast<const uint16_t*>(partials);
  const dim3 g256{unsigned(xcd_grid(gpr))}, g512{unsigned(xcd_grid((gpr + 1) / 2))};
#define RS_REDUCE(THREADS, DOUBLE, GRID)                                                         \
  shard_reduce_kernel<THREADS, DOUBLE><<<GRID, dim3(THREADS), 0, st>>>(                         \
      dev.tensors, n, dev.gran_first, P, row_stride, out, S, gpr, rank, world, inv_w)
  if (gpr >= 4096)
    RS_REDUCE(512, true, g512);
  else
    RS_REDUCE(256, false, g256);
#undef RS_REDUCE
  return launched();
}

int launch_block_quant(const DeviceTables& dev, int64_t item_off, int64_t item_count, const void* x,
                       uint8_t* codes, float* scales, void* const* batch, int batch_count,
                       int64_t elem_base, int64_t scale_off, hipStream_t st) {
  if (item_count == 0 || (batch && batch_count == 0)) return RS_OK;
  if (item_count < 0 || item_count > 0x7fffffffLL || batch_count < 0 || batch_count > 65535)
    return RS_EOVERFLOW;
  const int64_t work = item_count * (batch ? batch_count : 1);
  if (work > 0x7fffff00LL) return RS_EOVERFLOW;
  block_quant_kernel<<<dim3(unsigned(xcd_grid(work))), dim3(kQuantThreads), 0, st>>>(
      dev.tensors, dev.items, item_off, static_cast<const uint16_t*>(x), codes, scales, batch,
      batch_count, elem_base, scale_off, item_count);
  return launched();
}

int launch_dequant_unpack(bool f32_out, const DeviceTables& dev, int n, int64_t n_payload_gran,
                          const uint8_t* codes, const float* scales, void* const* ptrs, int64_t S,
                          int64_t gpr, hipStream_t st) {
  if (n_payload_gran == 0) return RS_OK;
  if (n_payload_gran < 0 || n_payload_gran > 0x7fffffffLL) return RS_EOVERFLOW;
  const dim3 g{unsigned(n_payload_gran)}, b{unsigned(kDequantThreads)};
  if (f32_out)
    dequant_unpack_kernel<true><<<g, b, 0, st>>>(dev.tensors, n, dev.gran_first, dev.payload_gran,
                                                 codes, scales, ptrs, S, gpr);
  else
    dequant_unpack_kernel<false><<<g, b, 0, st>>>(dev.tensors, n, dev.gran_first, dev.payload_gran,
                                                  codes, scales, ptrs, S, gpr);
  return launched();
}

int launch_adam8_step(const DeviceTables& dev, int64_t item_off, int64_t item_count, const float* grad,
                      float* master, void* param_bf16, int8_t* m_codes, uint8_t* v_codes,
                      float* m_absmax, float* v_absmax, void* const* batch, int batch_count,
                      int64_t elem_base, int64_t state_off, const Adam8Consts& c, hipStream_t st) {
  if (item_count == 0 || (batch && batch_count == 0)) return RS_OK;
  if (item_count < 0 || batch_count < 0) return RS_EOVERFLOW;
  const int64_t work = item_count * (batch ? batch_count : 1);
  if (work > 0x7fffff00LL) return RS_EOVERFLOW;
  adam8_step_kernel<<<dim3(unsigned(xcd_grid(work))), dim3(kStateThreads), 0, st>>>(
      dev.tensors, dev.state_items, item_off, item_count, grad, master,
      static_cast<uint16_t*>(param_bf16), reinterpret_cast<uint8_t*>(m_codes), v_codes, m_absmax,
      v_absmax, batch, batch_count, elem_base, state_off, c);
  return launched();
}

int launch_copy_probe(void* dst, const void* src, int64_t bytes, hipStream_t st) {
  const int64_t nvec = bytes / 16;
  const int64_t grid = (nvec + kCopyThreads - 1) / kCopyThreads;
  if (grid == 0) return RS_OK;
  if (grid > 0x7fffffffLL) return RS_EOVERFLOW;
  copy_probe_kernel<<<dim3(unsigned(grid)), dim3(kCopyThreads), 0, st>>>(
      static_cast<const u32x4*>(src), static_cast<u32x4*>(dst), nvec);
  return launched();
}

}  // namespace rs
