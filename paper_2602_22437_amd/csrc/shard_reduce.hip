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
    int64_t gpr, int rank, int W, float inv_w, void* const* __restrict__ batch, int batch_count,
    unsigned blocks_per_unit) {
  // with 512 lanes, waves 0-3 take the even granule of the pair, waves 4-7 the odd one
  const int half = __builtin_amdgcn_readfirstlane(int(threadIdx.x) / kThreads);  // wave-uniform
  int64_t blk = xcd_chunked(blockIdx.x, kXcdChunk);
  if (batch) {
    // the same region of batch_count units, their blocks end to end in one flat grid;
    // batch = [partials | out] pointers
    const unsigned u = unsigned(blk) / blocks_per_unit;   // both below 2^31: a 32-bit division
    if (u >= unsigned(batch_count)) return;
    blk -= int64_t(u) * blocks_per_unit;
    P = static_cast<const uint16_t*>(batch[u]);
    out = static_cast<float*>(batch[batch_count + u]);
  }
  const int64_t j = blk * (kReduceThreads / kThreads) + half;
  if (j >= gpr) return;
  const int64_t i0 = j * kGranule;
  const int64_t d0 = int64_t(rank) * S + i0;
  const int len = int(min(int64_t(kGranule), S - i0));
  const int lane_off = (threadIdx.x % kThreads) * 8;
  if (lane_off >= len) return;
  const int64_t d = d0 + lane_off;
  float* o = out + i0 + lane_off;

  // payload mask of this lane's 8 elements; a granule flagged as lying wholly inside one tensor
  // (nearly all of them) needs no further table read
  const int entry = gran_first[int64_t(rank) * gpr + j];
  const int t0 = entry & ~kGranWhole;
  unsigned mask = 0xffu;
  bool empty = t0 >= n;
  if (!empty && !(entry & kGranWhole)) {
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
                        float* out, int64_t S, int64_t gpr, int rank, int rows, void* const* batch,
                        int batch_count, hipStream_t st) {
  if (gpr <= 0 || gpr > 0x7fffffffLL) return RS_EOVERFLOW;
  if (batch && batch_count == 0) return RS_OK;
  if (batch_count < 0 || batch_count > 65535) return RS_EOVERFLOW;
  const float inv_w = 1.0f / float(rows);
  const uint16_t* P = static_cast<const uint16_t*>(partials);
  // the wide shape (two granules per workgroup, next rows in flight) pays once the launch is
  // long enough; the sums are the same either way
  const bool wide = gpr * (batch ? batch_count : 1) >= 4096;
  const int64_t blocks_per_unit = wide ? (gpr + 1) / 2 : gpr;
  const int64_t work = blocks_per_unit * (batch ? batch_count : 1);
  if (work > 0x7fffff00LL) return RS_EOVERFLOW;
  const dim3 grid{unsigned(xcd_grid(work))};
#define RS_REDUCE(THREADS, DOUBLE)                                                               \
  shard_reduce_kernel<THREADS, DOUBLE><<<grid, dim3(THREADS), 0, st>>>(                         \
      dev.tensors, n, dev.gran_first, P, row_stride, out, S, gpr, rank, rows, inv_w, batch,     \
      batch_count, unsigned(blocks_per_unit))
  if (wide)
    RS_REDUCE(512, true);
  else
    RS_REDUCE(256, false);
#undef RS_REDUCE
  return launched();
}

}  // namespace rs
