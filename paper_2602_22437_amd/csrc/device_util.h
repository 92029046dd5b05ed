// Device-side helpers shared by the kernel files: 16-byte vector accesses, the XCD-aware block
// index remap, DPP maxima, bf16 packing, and exact division by a shared divisor.
#pragma once
#include <hip/hip_runtime.h>

#include "rs_internal.h"
#include "rs_launch.h"

namespace rs {

typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef unsigned int u32x2 __attribute__((ext_vector_type(2)));

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

// Maximum of an unsigned value (or the bit pattern of a non-negative float) over each row of 16
// lanes, delivered to every lane of the row: four rotate-within-row DPP steps, no LDS traffic.
template <int kCtrl>
__device__ __forceinline__ unsigned dpp_max_step(unsigned v) {
  return max(v, unsigned(__builtin_amdgcn_update_dpp(0, int(v), kCtrl, 0xf, 0xf, false)));
}
__device__ __forceinline__ unsigned row16_max(unsigned v) {
  v = dpp_max_step<0x121>(v);   // row_ror:1
  v = dpp_max_step<0x122>(v);   // row_ror:2
  v = dpp_max_step<0x124>(v);   // row_ror:4
  return dpp_max_step<0x128>(v);   // row_ror:8
}
// the same over the whole wavefront, as a wave-uniform value
__device__ __forceinline__ unsigned wave_max(unsigned v) {
  v = row16_max(v);
  const unsigned a = __builtin_amdgcn_readlane(int(v), 0), b = __builtin_amdgcn_readlane(int(v), 16);
  const unsigned c = __builtin_amdgcn_readlane(int(v), 32), d = __builtin_amdgcn_readlane(int(v), 48);
  return max(max(a, b), max(c, d));
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

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// two fp32 -> packed bf16 pair, round to nearest even (one v_cvt_pk_bf16_f32 on gfx950)
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  return __builtin_bit_cast(unsigned, __builtin_convertvector(f32x2{lo, hi}, bf16x2));
}
__device__ __forceinline__ float bf16_lo(unsigned packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(unsigned packed) { return __uint_as_float(packed & 0xffff0000u); }

// The correctly rounded fp32 quotient x / b for many dividends x that share the divisor b (a
// block's scale or quantisation step, a constant of the optimiser), by way of double precision:
// RN32(RN64(x * rd)) with rd = RN64(1 / b).  Why this is RN32(x / b) exactly: let m be a midpoint
// between neighbouring fp32 values near y = x / b, where fp32 values are 2^(E-23) apart.  With x
// and b fp32 (24-bit significands), x - m * b is an integer multiple of 2^(E + e_b - 47), and it
// is never zero because m * b has at least 25 significant bits; so y lies at least 2^(E-48) from
// every midpoint.  The double product is within 2^(E-50) of y, falls on the same side of every
// midpoint, and its conversion to fp32 rounds it as y would be rounded.  No range restrictions
// (doubles neither over- nor underflow on fp32 inputs), -0 stays -0, and three full-rate
// operations per element instead of the twelve or so of the IEEE division sequence.
// rd need not be the correctly rounded reciprocal: the argument above leaves room for a relative
// error of 2^-50 in it.  The hardware estimate refined by two Newton steps is within 2^-52 for
// any estimate good to 2^-13 or better (the error squares in each step), at 5 operations instead
// of the twenty or so of a double-precision division.  b is a non-negative fp32 number: as a
// double it is zero or normal, and so is its reciprocal.  b == 0 gives +inf as the division would.
__device__ __forceinline__ double shared_reciprocal(float b) {
  const double d = double(b);
  double r = __builtin_amdgcn_rcp(d);
  r = __builtin_fma(__builtin_fma(-d, r, 1.0), r, r);
  r = __builtin_fma(__builtin_fma(-d, r, 1.0), r, r);
  return b == 0.0f ? __builtin_inf() : r;
}
__device__ __forceinline__ float exact_quotient(float x, double rd) { return float(double(x) * rd); }

// Correctly rounded fp32 square root of x >= 0 from the hardware's 1-ulp estimate s: the true root
// rounds to s - 1 ulp exactly when x <= s * (s - 1 ulp) (the product stands for the square of the
// midpoint; x - s * (s - 1 ulp) is a whole multiple of ulp(s)^2, so the quarter-ulp^2 between the
// two cannot matter), to s + 1 ulp when x > s * (s + 1 ulp), both residuals exact in one FMA each.
// Zero comes out as zero (the lower neighbour is a NaN pattern, its test false).  Valid for zero
// and for x >= 2^-100 (the residuals are multiples of ulp(s)^2 >= 2^-146, exactly representable;
// the products inside the FMAs are exact, so large x cannot overflow them); below, the
// estimate's own input scaling would be needed and the compiler's sequence is taken instead (a
// branch uniform across the wavefront, all but never taken).
__device__ __forceinline__ float exact_sqrt(float x) {
  // out of range: 0 < x < 2^-100, as one unsigned comparison of the bit pattern
  const bool low = (__float_as_uint(x) - 1u) < ((27u << 23) - 1u);
  if (__builtin_amdgcn_ballot_w64(low) != 0) return __builtin_sqrtf(x);
  const float s = __builtin_amdgcn_sqrtf(x);
  const float dn = __uint_as_float(__float_as_uint(s) - 1u), up = __uint_as_float(__float_as_uint(s) + 1u);
  const float t_dn = __builtin_fmaf(-dn, s, x), t_up = __builtin_fmaf(-up, s, x);
  float r = t_dn <= 0.0f ? dn : s;
  r = t_up > 0.0f ? up : r;
  return r;
}

// status of the launch just enqueued
static inline int launched() { return hipGetLastError() == hipSuccess ? RS_OK : RS_EHIP; }

}  // namespace rs
