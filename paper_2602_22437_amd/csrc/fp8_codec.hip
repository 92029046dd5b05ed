// block_quant and dequant_unpack: block-wise FP8 E4M3 of the local shard and its inverse into
// per-tensor storage (gfx950, wave64; hardware OCP FP8 converts).
#include "device_util.h"
#include "quant_items.h"

namespace rs {

typedef unsigned short u16x2 __attribute__((ext_vector_type(2)));

// bf16 magnitudes order like their 15-bit patterns; both halves of a word at once
// (v_and_b32 + v_pk_max_u16)
__device__ __forceinline__ u16x2 abs_pair(unsigned packed) {
  return __builtin_bit_cast(u16x2, packed & 0x7fff7fffu);
}

// largest 15-bit magnitude pattern among the 8 bf16 values of a vector
__device__ __forceinline__ unsigned abs_max8(const u32x4 v) {
  const u16x2 ab = __builtin_elementwise_max(abs_pair(v.x), abs_pair(v.y));
  const u16x2 cd = __builtin_elementwise_max(abs_pair(v.z), abs_pair(v.w));
  const unsigned mx = __builtin_bit_cast(unsigned, __builtin_elementwise_max(ab, cd));
  return max(mx & 0xffffu, mx >> 16);
}

// scale = amax / 448, correctly rounded (one fp32 division per block)
__device__ __forceinline__ float scale_of(unsigned amax_bits) {
  return __uint_as_float(amax_bits << 16) / kE4M3Max;
}

// codes of 8 bf16 values of a block: E4M3(clamp(RN(x / scale))), the quotient by way of the
// block's double-precision reciprocal (exact_quotient in device_util.h), hardware RNE convert
__device__ __forceinline__ u32x2 quant8(const u32x4 v, double rd) {
  const float x[8] = {bf16_lo(v.x), bf16_hi(v.x), bf16_lo(v.y), bf16_hi(v.y),
                      bf16_lo(v.z), bf16_hi(v.z), bf16_lo(v.w), bf16_hi(v.w)};
  float q[8];
#pragma unroll
  for (int j = 0; j < 8; ++j)
    q[j] = __builtin_amdgcn_fmed3f(exact_quotient(x[j], rd), -kE4M3Max, kE4M3Max);
  u32x2 c;
  c.x = unsigned(__builtin_amdgcn_cvt_pk_fp8_f32(q[2], q[3], __builtin_amdgcn_cvt_pk_fp8_f32(q[0], q[1], 0, false), true));
  c.y = unsigned(__builtin_amdgcn_cvt_pk_fp8_f32(q[6], q[7], __builtin_amdgcn_cvt_pk_fp8_f32(q[4], q[5], 0, false), true));
  return c;
}

// One work item whose rows are 16-byte structured: 128 slots of 128 elements, slot s at
// x + s * pitch.  kTile: one scale for the whole item (a 128x128 tile, of which `rows` x `cols`
// exist when kMask; cols is a multiple of 8); otherwise one scale per slot (128 consecutive
// 1x128 blocks), written to scales[slot].
template <bool kTile, bool kMask>
__device__ __forceinline__ void quant_lean_item(const uint16_t* __restrict__ x,
                                                uint8_t* __restrict__ codes, int64_t pitch,
                                                float* __restrict__ scales, unsigned* wave_max_lds,
                                                int rows, int cols) {
  const int tid = threadIdx.x;
  const int64_t lane_off = int64_t(tid >> 4) * pitch + (tid & 15) * 8;
  const int64_t step = int64_t(kQuantRowStep) * pitch;
  u32x4 v[kQuantLoads];
  bool on[kQuantLoads];
#pragma unroll
  for (int i = 0; i < kQuantLoads; ++i) {
    on[i] = !kMask || (((tid & 15) * 8 < cols) & ((tid >> 4) + kQuantRowStep * i < rows));
    v[i] = u32x4{0, 0, 0, 0};
    if (on[i]) v[i] = ld16(x + lane_off + i * step);
  }
  unsigned m[kQuantLoads];
#pragma unroll
  for (int i = 0; i < kQuantLoads; ++i) m[i] = abs_max8(v[i]);
  double rd[kQuantLoads];
  if (kTile) {
    unsigned a = wave_max(max(max(m[0], m[1]), max(m[2], m[3])));
    if ((tid & 63) == 0) wave_max_lds[tid >> 6] = a;
    __syncthreads();
    a = wave_max_lds[0];
#pragma unroll
    for (int w = 1; w < kQuantThreads / 64; ++w) a = max(a, wave_max_lds[w]);
    const float sc = scale_of(a);
    if (tid == 0) scales[0] = sc;
    const double r = shared_reciprocal(sc);
#pragma unroll
    for (int i = 0; i < kQuantLoads; ++i) {
      m[i] = a;
      rd[i] = r;
    }
  } else {
#pragma unroll
    for (int i = 0; i < kQuantLoads; ++i) {
      m[i] = row16_max(m[i]);
      const float sc = scale_of(m[i]);
      if ((tid & 15) == 0) scales[(tid >> 4) + kQuantRowStep * i] = sc;
      rd[i] = shared_reciprocal(sc);
    }
  }
#pragma unroll
  for (int i = 0; i < kQuantLoads; ++i) {
    if (!on[i]) continue;
    u32x2 c{0, 0};
    if (m[i] != 0) c = quant8(v[i], rd[i]);
    st8(codes + lane_off + i * step, c);
  }
}

// -------------------------------------------------------------------------------------------
// block_quant: amax per block (wavefront shuffles, LDS across the 8 waves of a tile),
// scale = amax / 448, codes = E4M3(clamp(x / scale)) with the hardware RNE convert.
// x / codes are addressed relative to elem_base (0 or rank * S), scales to scale_off.
// -------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kQuantThreads) void block_quant_kernel(
    const TensorDev* __restrict__ T, const QItem* __restrict__ items, int64_t item_off,
    const uint16_t* __restrict__ x_one, uint8_t* __restrict__ codes_one,
    float* __restrict__ scales_one, void* const* __restrict__ batch, int batch_count,
    int64_t elem_base, int64_t scale_off, int64_t item_count) {
  __shared__ unsigned wave_max_lds[kQuantThreads / 64];
  // batched launch: batch = [shards | codes | scales] pointers of batch_count units
  const uint16_t* __restrict__ x = x_one;
  uint8_t* __restrict__ codes = codes_one;
  float* __restrict__ scales = scales_one;
  // adjacent tiles of a row of tiles share DRAM pages and cache lines: keep them on one XCD
  int64_t idx = xcd_chunked(blockIdx.x, kXcdChunk);
  if (batch) {
    // the units' item ranges are laid end to end in one flat grid: no idle tail per unit
    const int64_t u = unsigned(idx) / unsigned(item_count);   // both below 2^31: a 32-bit division
    if (u >= batch_count) return;
    idx -= u * item_count;
    x = static_cast<const uint16_t*>(batch[u]);
    codes = static_cast<uint8_t*>(batch[batch_count + u]);
    scales = static_cast<float*>(batch[2 * batch_count + u]);
  } else if (idx >= item_count) {
    return;
  }
  const QItem it = items[item_off + idx];
  if (it.tensor < 0) {
    zero_fill_bytes(codes + (it.first - elem_base), it.count, kQuantThreads);
    return;
  }
  // Items whose rows are 16-byte structured (nearly all of them) need nothing but their own
  // record: no per-slot bookkeeping, straight-line loads, one reduction, straight-line stores.
  if (it.lean != 0) {
    const int64_t off = it.elem - elem_base;
    float* const sc = scales + (it.scale - scale_off);
    if (it.lean == 2)
      quant_lean_item<false, false>(x + off, codes + off, 128, sc, wave_max_lds, 128, 128);
    else if (it.rows == 128 && it.cols == 128)
      quant_lean_item<true, false>(x + off, codes + off, it.pitch, sc, wave_max_lds, 128, 128);
    else
      quant_lean_item<true, true>(x + off, codes + off, it.pitch, sc, wave_max_lds, it.rows, it.cols);
    return;
  }
  // tensors without that structure (odd row pitches, unaligned starts, ragged runs)
  const TensorDev t = T[it.tensor];
  const bool tile = (t.flags & kFlagTile) != 0;
  const bool vec = (t.flags & kFlagVec) != 0;
  const int tid = threadIdx.x;
  const int r_in = tid >> 4, col0 = (tid & 15) * 8;
  const int64_t base = t.ell - elem_base;

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
  for (int i = 0; i < kQuantLoads; ++i) m[i] = abs_max8(v[i]);
  double rd[kQuantLoads];
  if (tile) {
    unsigned a = wave_max(max(max(m[0], m[1]), max(m[2], m[3])));
    if ((tid & 63) == 0) wave_max_lds[tid >> 6] = a;
    __syncthreads();
    a = wave_max_lds[0];
#pragma unroll
    for (int w = 1; w < kQuantThreads / 64; ++w) a = max(a, wave_max_lds[w]);
    const float sc = scale_of(a);
    const double r = shared_reciprocal(sc);
#pragma unroll
    for (int i = 0; i < kQuantLoads; ++i) {
      m[i] = a;
      rd[i] = r;
    }
    if (tid == 0) scales[t.scale_base + it.first * t.nbc + it.count - scale_off] = sc;
  } else {
#pragma unroll
    for (int i = 0; i < kQuantLoads; ++i) {
      m[i] = row16_max(m[i]);
      const float sc = scale_of(m[i]);
      rd[i] = shared_reciprocal(sc);
      if ((tid & 15) == 0 && r_in + kQuantRowStep * i < it.count)
        scales[t.scale_base + sl[i].blk - scale_off] = sc;
    }
  }

#pragma unroll
  for (int i = 0; i < kQuantLoads; ++i) {
    if (sl[i].ncol == 0) continue;
    u32x2 c{0, 0};
    if (m[i] != 0) c = quant8(v[i], rd[i]);
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
// Buffer-driven like ragged_pack: one workgroup of kDequantThreads lanes (one wavefront for bf16
// output, two for fp32) per granule that holds payload; a lane converts 8 codes (one 8-byte
// load, one 16-byte store) in each quarter of the granule, or 4 codes per 16-byte fp32 store.
// No block-wide step is needed, only the block's scale.
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


// kF32: the tensors are fp32 (value * scale, no further rounding) instead of bf16
template <bool kF32, int kDequantThreads = 64>
__global__ __launch_bounds__(kDequantThreads) void dequant_unpack_kernel(
    const TensorDev* __restrict__ T, int n, const GranRef* __restrict__ granules,
    const uint8_t* __restrict__ codes,
    const float* __restrict__ scales, void* const* __restrict__ ptrs, int64_t S, int64_t gpr,
    int64_t region_stride) {
  // one 8-byte read: the granule and its first tensor (a payload granule: t0 < n)
  const long long packed = reinterpret_cast<const long long*>(granules)[blockIdx.x];
  const int t0 = int32_t(packed >> 32);
  // the tensor's record and base pointer are requested at once, ahead of the index arithmetic
  const TensorDev t = T[t0];
  void* const tensor = ptrs[t0];
  const unsigned gid = unsigned(packed);             // granule ids and gpr fit 31 bits
  const unsigned k = gid / unsigned(gpr);
  const int64_t i0 = int64_t(gid - k * unsigned(gpr)) * kGranule;
  const int64_t d0 = k * S + i0;            // logical buffer position: what the tables speak of
  // where the granule's codes live: rank regions are region_stride bytes apart (S in a plain buffer)
  const uint8_t* __restrict__ const src = codes + k * region_stride + i0;
  const int len = int(min(int64_t(kGranule), S - i0));
  // A lane converts kGroup codes per access so that its store is one 16-byte vector and a
  // wavefront's stores are contiguous: 8 codes -> 8 bf16, or 4 codes -> 4 fp32.
  constexpr int kGroup = kF32 ? 4 : 8;
  constexpr int kStep = kDequantThreads * kGroup;   // codes per access of the workgroup
  constexpr int kParts = kGranule / kStep;
  const int lane = threadIdx.x * kGroup;

  {
    uint16_t* out = reinterpret_cast<uint16_t*>(tensor);
    float* out32 = reinterpret_cast<float*>(tensor);
    // one round of table reads, one branch
    const bool inside = (t.ell <= d0) & (d0 + len <= t.ell + t.e);
    const bool structured = ((t.flags & kFlagVec) != 0) & ((reinterpret_cast<uintptr_t>(out) & 15) == 0) &
                            (t.cols < (int64_t(1) << 30));
    if (inside & structured) {
      // The whole granule lies in one tensor whose rows keep every 8-element group inside one
      // row and one block.  (row, col) of the granule's first element once per workgroup
      // (exact: a double holds any element index below 2^53), then 32-bit steps per lane.
      const int64_t first = d0 - t.ell;
      int64_t row0 = int64_t(double(first) / double(t.cols));
      int64_t col0 = first - row0 * t.cols;
      if (col0 < 0) { col0 += t.cols; --row0; }
      if (col0 >= t.cols) { col0 -= t.cols; ++row0; }
      const unsigned C = unsigned(t.cols);
      const bool tile = (t.flags & kFlagTile) != 0;
      const bool contig = (t.flags & kFlagContig) && !tile;
      // scale of the granule's first element, the same for the whole workgroup: scalar arithmetic
      const int64_t row0u = (int64_t(__builtin_amdgcn_readfirstlane(int(row0 >> 32))) << 32) |
                            unsigned(__builtin_amdgcn_readfirstlane(int(row0)));
      const float* __restrict__ const sc0 =
          scales + t.scale_base + (contig ? (first >> 7) : (tile ? (row0u >> 7) : row0u) * t.nbc);
      const unsigned row_in_tile = tile ? unsigned(row0u) & 127u : 0u;
      // this lane's first group: rows past row0 and column, by one 32-bit division; the following
      // parts are kStep elements further on, which is at most one row when rows are that long
      unsigned cc = unsigned(col0) + unsigned(lane), dr = 0;
      if (!contig) {
        dr = cc / C;
        cc -= dr * C;
      }
      const bool long_rows = C >= unsigned(kStep);
      u32x2 c[kParts];
      float sc[kParts];
      bool on[kParts];
#pragma unroll
      for (int h = 0; h < kParts; ++h) {
        const int lo = h * kStep + lane;
        on[h] = lo < len;
        if (on[h]) {
          if (kF32)
            c[h] = u32x2{__builtin_nontemporal_load(reinterpret_cast<const unsigned*>(src + lo)), 0};
          else
            c[h] = ld8(src + lo);
          unsigned sidx;
          if (contig)
            sidx = ((unsigned(first) & 127u) + unsigned(lo)) >> 7;   // consecutive runs of 128 elements
          else
            sidx = (tile ? ((row_in_tile + dr) >> 7) : dr) * unsigned(t.nbc) + (cc >> 7);
          sc[h] = sc0[sidx];
        }
        if (!contig && h + 1 < kParts) {     // on to the next part
          if (long_rows) {
            cc += kStep;
            if (cc >= C) {
              cc -= C;
              ++dr;
            }
          } else {
            const unsigned c2 = cc + kStep, k2 = c2 / C;
            dr += k2;
            cc = c2 - k2 * C;
          }
        }
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
      const auto f = __builtin_amdgcn_cvt_pk_f32_fp8(int(src[lo + q]), false);
      if (kF32)
        reinterpret_cast<float*>(ptrs[s])[i] = f[0] * scale;
      else
        reinterpret_cast<uint16_t*>(ptrs[s])[i] = uint16_t(bf16_rne(f[0] * scale));
    }
  }
}

// -------------------------------------------------------------------------------------------
// launchers (host)
// -------------------------------------------------------------------------------------------
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
                          int64_t gpr, int64_t region_stride, hipStream_t st) {
  if (n_payload_gran == 0) return RS_OK;
  if (n_payload_gran < 0 || n_payload_gran > 0x7fffffffLL) return RS_EOVERFLOW;
  const dim3 g{unsigned(n_payload_gran)};
  // fp32 output is four fifths writes: two wavefronts per granule measured 3 % faster than one
  // (configurations 2 and 4; no change on 5), four 5 % slower
  if (f32_out)
    dequant_unpack_kernel<true, 128><<<g, dim3(128), 0, st>>>(dev.tensors, n, dev.payload_gran,
                                                             codes, scales, ptrs, S, gpr, region_stride);
  else
    dequant_unpack_kernel<false><<<g, dim3(64), 0, st>>>(dev.tensors, n, dev.payload_gran,
                                                  codes, scales, ptrs, S, gpr, region_stride);
  return launched();
}

}  // namespace rs
