// shard_reduce: the arithmetic of the gradient ReduceScatter as one rank sees it (gfx950, wave64).
#include "device_util.h"
#include "reduce_order.h"

namespace rs {

constexpr int kThreads = 256;  // lanes per granule

// -------------------------------------------------------------------------------------------
// shard_reduce: out[i] = (1/W) * sum_w P[w][i] on the payload of one rank region, 0 on padding.
// Each lane owns 8 consecutive elements and walks the W rows; rows are spread over 8
// accumulator sets (row w -> set w mod 8) that are combined pairwise at the end, so the
// summation order is fixed and the rounding error grows with W/8 + 3, not W.
// -------------------------------------------------------------------------------------------
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

  float sum[8], r[8];
  reduce_column<kDouble, true>(P + i0 + lane_off, row_stride, W, 8, sum);
#pragma unroll
  for (int q = 0; q < 8; ++q) r[q] = (mask >> q) & 1u ? sum[q] * inv_w : 0.0f;
  st16(o, u32x4{__float_as_uint(r[0]), __float_as_uint(r[1]), __float_as_uint(r[2]),
                __float_as_uint(r[3])});
  st16(o + 4, u32x4{__float_as_uint(r[4]), __float_as_uint(r[5]), __float_as_uint(r[6]),
                    __float_as_uint(r[7])});
}

// -------------------------------------------------------------------------------------------
// launcher (host)
// -------------------------------------------------------------------------------------------
int launch_shard_reduce(const DeviceTables& dev, int n, const void* partials, int64_t row_stride,
                        float* out, int64_t S, int64_t gpr, int rank, int rows, hipStream_t st) {
  if (gpr <= 0 || gpr > 0x7fffffffLL) return RS_EOVERFLOW;
  const float inv_w = 1.0f / float(rows);
  const uint16_t* P = static_cast<const uint16_t*>(partials);
  const dim3 g256{unsigned(xcd_grid(gpr))}, g512{unsigned(xcd_grid((gpr + 1) / 2))};
#define RS_REDUCE(THREADS, DOUBLE, GRID)                                                         \
  shard_reduce_kernel<THREADS, DOUBLE><<<GRID, dim3(THREADS), 0, st>>>(                         \
      dev.tensors, n, dev.gran_first, P, row_stride, out, S, gpr, rank, rows, inv_w)
  if (gpr >= 4096)
    RS_REDUCE(512, true, g512);
  else
    RS_REDUCE(256, false, g256);
#undef RS_REDUCE
  return launched();
}

}  // namespace rs
