// reduce_quant: shard_reduce and block_quant fused (gfx950, wave64).  The fp32 mean of the W
// partials is formed in registers, block by block, and leaves the chip as FP8 codes and scales
// only (optionally also as fp32, for a caller that needs both).
#include "device_util.h"
#include "quant_items.h"
#include "reduce_order.h"

namespace rs {

// One workgroup per quantisation work item of the rank, as in block_quant: lane (tid / 16,
// tid % 16) owns 8 elements of slots tid / 16 + 32 i, i = 0..3.  For each of its four slots in
// turn the lane walks the W rows with the summation order of shard_reduce (same code, same
// bits), which keeps eight 16-byte loads in flight per lane; the block maximum and the codes
// then follow block_quant's steps on fp32 values (prefetching the next eight rows, or the next
// slot's first rows, while a group is added was measured and gained nothing):
//   scale = amax / 448 (fp32 division), code = E4M3(clamp(mean / scale)) (correctly rounded
//   division, hardware RNE convert).  A block whose scale underflows to zero (amax below
//   2^-140, which no bf16 input reaches) is stored as a zero block.
template <bool kVec>
__device__ __forceinline__ void slot_mean(const uint16_t* p, int64_t row_stride, int W, float inv_w,
                                          int ncol, float (&r)[8]) {
  float sum[8];
  reduce_column<false, kVec>(p, row_stride, W, ncol, sum);
#pragma unroll
  for (int q = 0; q < 8; ++q) r[q] = q < ncol ? sum[q] * inv_w : 0.0f;
}

__device__ __forceinline__ unsigned quant4(float a, float b, float c, float e, double rd) {
  const float qa = __builtin_amdgcn_fmed3f(exact_quotient(a, rd), -kE4M3Max, kE4M3Max);
  const float qb = __builtin_amdgcn_fmed3f(exact_quotient(b, rd), -kE4M3Max, kE4M3Max);
  const float qc = __builtin_amdgcn_fmed3f(exact_quotient(c, rd), -kE4M3Max, kE4M3Max);
  const float qe = __builtin_amdgcn_fmed3f(exact_quotient(e, rd), -kE4M3Max, kE4M3Max);
  const int lo = __builtin_amdgcn_cvt_pk_fp8_f32(qa, qb, 0, false);
  return unsigned(__builtin_amdgcn_cvt_pk_fp8_f32(qc, qe, lo, true));
}

__global__ __launch_bounds__(kQuantThreads) void reduce_quant_kernel(
    const TensorDev* __restrict__ T, const QItem* __restrict__ items, int64_t item_off,
    int64_t item_count, const uint16_t* __restrict__ P_one, int64_t row_stride,
    uint8_t* __restrict__ codes_one, float* __restrict__ scales_one, float* __restrict__ mean_one,
    void* const* __restrict__ batch_in, void* const* __restrict__ batch_out, int batch_count,
    int write_means, int64_t elem_base, int64_t scale_off, int W, float inv_w) {
  __shared__ unsigned wave_max_lds[kQuantThreads / 64];
  const uint16_t* __restrict__ P = P_one;
  uint8_t* __restrict__ codes = codes_one;
  float* __restrict__ scales = scales_one;
  float* __restrict__ mean_out = mean_one;
  int64_t idx = xcd_chunked(blockIdx.x, kXcdChunk);
  if (batch_in) {
    // the units' item ranges end to end in one flat grid; batch_in = [partials | means],
    // batch_out = [shards (unused) | codes | scales], batch_count pointers each
    const int64_t u = unsigned(idx) / unsigned(item_count);   // both below 2^31
    if (u >= batch_count) return;
    idx -= u * item_count;
    P = static_cast<const uint16_t*>(batch_in[u]);
    mean_out = write_means ? static_cast<float*>(batch_in[batch_count + u]) : nullptr;
    codes = static_cast<uint8_t*>(batch_out[batch_count + u]);
    scales = static_cast<float*>(batch_out[2 * batch_count + u]);
  } else if (idx >= item_count) {
    return;
  }
  const QItem it = items[item_off + idx];
  const int tid = threadIdx.x;
  if (it.tensor < 0) {   // padding of the region: zero codes, zero mean
    const int64_t off = it.first - elem_base;
    zero_fill_bytes(codes + off, it.count, kQuantThreads);
    if (mean_out)
      for (int i = tid; i < it.count; i += kQuantThreads) mean_out[off + i] = 0.0f;
    return;
  }
  const TensorDev t = T[it.tensor];
  const bool tile = (t.flags & kFlagTile) != 0;
  const bool vec = (t.flags & kFlagVec) != 0;
  const int r_in = tid >> 4, col0 = (tid & 15) * 8;
  const int64_t base = t.ell - elem_base;

  Slot sl[kQuantLoads];
  float r[kQuantLoads][8];
#pragma unroll
  for (int i = 0; i < kQuantLoads; ++i) {
    sl[i] = tile ? tile_slot(t, it.first, it.count, r_in + kQuantRowStep * i, col0)
                 : run_slot(t, it.first, it.count, r_in + kQuantRowStep * i, col0);
#pragma unroll
    for (int q = 0; q < 8; ++q) r[i][q] = 0.0f;
    if (sl[i].ncol == 0) continue;
    const uint16_t* p = P + base + sl[i].off;
    // a 16-byte load may take in elements of the next row or tensor: they are summed and dropped
    if (vec)
      slot_mean<true>(p, row_stride, W, inv_w, sl[i].ncol, r[i]);
    else
      slot_mean<false>(p, row_stride, W, inv_w, sl[i].ncol, r[i]);
  }

  // block maximum of |mean|: fp32 magnitudes order like their 31-bit patterns
  unsigned m[kQuantLoads];
#pragma unroll
  for (int i = 0; i < kQuantLoads; ++i) {
    unsigned a = 0;
#pragma unroll
    for (int q = 0; q < 8; ++q) a = max(a, __float_as_uint(r[i][q]) & 0x7fffffffu);
    m[i] = a;
  }
  float scale[kQuantLoads];
  if (tile) {
    unsigned a = wave_max(max(max(m[0], m[1]), max(m[2], m[3])));
    if ((tid & 63) == 0) wave_max_lds[tid >> 6] = a;
    __syncthreads();
    a = wave_max_lds[0];
#pragma unroll
    for (int w = 1; w < kQuantThreads / 64; ++w) a = max(a, wave_max_lds[w]);
    const float s = __uint_as_float(a) / kE4M3Max;
#pragma unroll
    for (int i = 0; i < kQuantLoads; ++i) scale[i] = s;
    if (tid == 0) scales[t.scale_base + it.first * t.nbc + it.count - scale_off] = s;
  } else {
#pragma unroll
    for (int i = 0; i < kQuantLoads; ++i) {
      const unsigned a = row16_max(m[i]);
      scale[i] = __uint_as_float(a) / kE4M3Max;
      if ((tid & 15) == 0 && r_in + kQuantRowStep * i < it.count)
        scales[t.scale_base + sl[i].blk - scale_off] = scale[i];
    }
  }

#pragma unroll
  for (int i = 0; i < kQuantLoads; ++i) {
    if (sl[i].ncol == 0) continue;
    u32x2 c{0, 0};
    if (scale[i] != 0.0f) {
      const double d = shared_reciprocal(scale[i]);
      c.x = quant4(r[i][0], r[i][1], r[i][2], r[i][3], d);
      c.y = quant4(r[i][4], r[i][5], r[i][6], r[i][7], d);
    }
    const int64_t at = base + sl[i].off;
    if (vec && sl[i].ncol == 8) {
      st8(codes + at, c);
      if (mean_out) {
        st16(mean_out + at, u32x4{__float_as_uint(r[i][0]), __float_as_uint(r[i][1]),
                                  __float_as_uint(r[i][2]), __float_as_uint(r[i][3])});
        st16(mean_out + at + 4, u32x4{__float_as_uint(r[i][4]), __float_as_uint(r[i][5]),
                                      __float_as_uint(r[i][6]), __float_as_uint(r[i][7])});
      }
    } else {
#pragma unroll
      for (int q = 0; q < 8; ++q)
        if (q < sl[i].ncol) {
          codes[at + q] = uint8_t((q < 4 ? c.x : c.y) >> ((q & 3) * 8));
          if (mean_out) mean_out[at + q] = r[i][q];
        }
    }
  }
}

int launch_reduce_quant(const DeviceTables& dev, int64_t item_off, int64_t item_count,
                        const void* partials, int64_t row_stride, uint8_t* codes, float* scales,
                        float* mean_out, void* const* batch_in, void* const* batch_out,
                        int batch_count, bool write_means, int64_t elem_base, int64_t scale_off,
                        int world, hipStream_t st) {
  if (item_count == 0 || (batch_in && batch_count == 0)) return RS_OK;
  if (item_count < 0 || item_count > 0x7fffffffLL || batch_count < 0 || batch_count > 65535)
    return RS_EOVERFLOW;
  const int64_t work = item_count * (batch_in ? batch_count : 1);
  if (work > 0x7fffff00LL) return RS_EOVERFLOW;
  reduce_quant_kernel<<<dim3(unsigned(xcd_grid(work))), dim3(kQuantThreads), 0, st>>>(
      dev.tensors, dev.items, item_off, item_count, static_cast<const uint16_t*>(partials), row_stride,
      codes, scales, mean_out, batch_in, batch_out, batch_count, write_means ? 1 : 0, elem_base,
      scale_off, world, 1.0f / float(world));
  return launched();
}

}  // namespace rs
