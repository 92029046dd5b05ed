// adam8_step: AdamW on the local shard with block-wise 8-bit moments (gfx950, wave64).
#include "device_util.h"

namespace rs {

// -------------------------------------------------------------------------------------------
// adam8_step: AdamW on the local shard with block-wise 8-bit moments.
// A workgroup of 1024 lanes owns one state work item: 32 rows x 256 columns of a 2-D tensor (a
// row of eight 32x32 state tiles), or 64 runs of 128 elements (1-D tensors, matrices of one-row
// granularity) seen as 32 rows of 256 elements.  Lane (cq, rw) = (tid % 64, tid / 64) handles the 4 elements at column 4 * cq of
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
    const int run = 2 * row_in + (cq >> 5);   // run within the item; the item's 32 "rows" hold two each
    if (run < it.count) {
      const int64_t q = it.first + run;       // run index within the tensor
      int64_t elem, left;
      if (t.flags & kFlagContig) {            // 1-D, or rows that are whole runs: runs are back to back
        elem = q * 128 + 4 * (cq & 31);
        left = t.e - elem;
      } else {                                // the last run of every row is short
        const int64_t row = q / t.sbc;
        const int64_t col = (q - row * t.sbc) * 128 + 4 * (cq & 31);
        elem = row * t.cols + col;
        left = t.cols - col;
      }
      if (left > 0) {
        s.nv = int(min(int64_t(4), left));
        s.off = base + elem;
        s.blk = int(t.state_base + q - state_off);
      }
    }
  }
  return s;
}

// step = absmax / levels (levels 127 or 255), correctly rounded, by the shared-divisor quotient
// with the constant's reciprocal
__device__ __forceinline__ float quant_step(float absmax, float levels) {
  return exact_quotient(absmax, levels == 127.0f ? 1.0 / 127.0 : 1.0 / 255.0);
}

// Reciprocal of a block's quantisation step for exact_quotient; an all-zero block (absmax 0,
// step 0) gets 0, which turns every code of the block into 0.
__device__ __forceinline__ double step_reciprocal(float absmax, float levels) {
  return absmax == 0.0f ? 0.0 : shared_reciprocal(quant_step(absmax, levels));
}

// code = rint(x / step) clamped to [lo, hi]
__device__ __forceinline__ int state_code(float x, double step_rcp, float lo, float hi) {
  return int(__builtin_amdgcn_fmed3f(__builtin_rintf(exact_quotient(x, step_rcp)), lo, hi));
}

// maximum of non-negative floats over the 8 lanes of a 32-column state tile (lanes 8k .. 8k+7),
// in every lane: neighbour swap, pair swap, mirror within the 8 - three DPP steps
__device__ __forceinline__ float tile8_max(float v) {
  unsigned u = __float_as_uint(v);
  u = dpp_max_step<0xB1>(u);    // quad_perm [1,0,3,2]
  u = dpp_max_step<0x4E>(u);    // quad_perm [2,3,0,1]
  u = dpp_max_step<0x141>(u);   // row_half_mirror
  return __uint_as_float(u);
}
// the same over 32 lanes (a run of 128 elements): a row of 16 by rotations, then the other row
__device__ __forceinline__ float run32_max(float v) {
  const unsigned u = row16_max(__float_as_uint(v));
  return __uint_as_float(max(u, unsigned(__shfl_xor(int(u), 16))));
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
      const float root = exact_quotient(exact_sqrt(v[i][j]), c.bc2_sqrt_rcp);
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
    a = tile8_max(a);
    b = tile8_max(b);
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
      const float a = run32_max(mmax[i]), b = run32_max(vmax[i]);
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
    const double s1 = step_reciprocal(mmax[i], 127.0f), s2 = step_reciprocal(vmax[i], 255.0f);
    unsigned cm = 0, cv = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      cm |= (unsigned(state_code(m[i][j], s1, -127.0f, 127.0f)) & 0xffu) << (8 * j);
      cv |= (unsigned(state_code(v[i][j], s2, 0.0f, 255.0f)) & 0xffu) << (8 * j);
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
    const int64_t u = unsigned(idx) / unsigned(item_count);   // both below 2^31: a 32-bit division
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
  if (t.flags & kFlagStateRuns)
    adam8_item<false, false>(t, it, g, w, p, mc, vc, am, av, elem_base, state_off, c, tile_max);
  else if ((t.flags & kFlagVec4) && (it.first + 1) * 32 <= t.rows &&
           int64_t(it.count + 1) * kStateCols <= t.cols)
    adam8_item<true, true>(t, it, g, w, p, mc, vc, am, av, elem_base, state_off, c, tile_max);
  else
    adam8_item<true, false>(t, it, g, w, p, mc, vc, am, av, elem_base, state_off, c, tile_max);
}

// -------------------------------------------------------------------------------------------
// The 8-bit codec on its own, same work items and lane mapping as the step:
//   kQuant:  fp32 -> codes + absmax (the block maximum by shuffles and LDS, as in the step)
//   else:    codes + absmax -> fp32
// is_unsigned selects the second-moment map (0..255) instead of the first-moment one (-127..127).
// -------------------------------------------------------------------------------------------
template <bool kQuant, bool kTile>
__device__ __forceinline__ void state_codec_item(const TensorDev& t, const Item& it,
                                                 float* __restrict__ x, uint8_t* __restrict__ codes,
                                                 float* __restrict__ absmax, bool is_unsigned,
                                                 int64_t elem_base, int64_t state_off,
                                                 float (*tile_max)[kStateCols / 32]) {
  const int tid = threadIdx.x;
  const int cq = tid & 63, rw = tid >> 6;
  const bool vec = (t.flags & kFlagVec4) != 0;
  const int64_t base = t.ell - elem_base;
  const float levels = is_unsigned ? 255.0f : 127.0f;

  StateSlot sl[kStateSlots];
  float v[kStateSlots][4];
  float vmax[kStateSlots];
#pragma unroll
  for (int i = 0; i < kStateSlots; ++i) {
    sl[i] = state_slot<kTile>(t, it, rw + kStateWaves * i, cq, base, state_off);
    vmax[i] = 0.0f;
#pragma unroll
    for (int j = 0; j < 4; ++j) v[i][j] = 0.0f;
    if (sl[i].nv == 0) continue;
    if (kQuant) {
      if (vec && sl[i].nv == 4) {
        const u32x4 q = ld16(x + sl[i].off);
        v[i][0] = __uint_as_float(q.x);
        v[i][1] = __uint_as_float(q.y);
        v[i][2] = __uint_as_float(q.z);
        v[i][3] = __uint_as_float(q.w);
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (j < sl[i].nv) v[i][j] = x[sl[i].off + j];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) vmax[i] = fmaxf(vmax[i], is_unsigned ? v[i][j] : __builtin_fabsf(v[i][j]));
    } else {
      unsigned c = 0;
      if (vec && sl[i].nv == 4) {
        c = __builtin_nontemporal_load(reinterpret_cast<const unsigned*>(codes + sl[i].off));
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (j < sl[i].nv) c |= unsigned(codes[sl[i].off + j]) << (8 * j);
      }
      const float step = quant_step(absmax[sl[i].blk], levels);
      float out[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const unsigned b = (c >> (8 * j)) & 0xffu;
        out[j] = (is_unsigned ? float(b) : float(int(int8_t(b)))) * step;
      }
      if (vec && sl[i].nv == 4) {
        st16(x + sl[i].off, u32x4{__float_as_uint(out[0]), __float_as_uint(out[1]),
                                  __float_as_uint(out[2]), __float_as_uint(out[3])});
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (j < sl[i].nv) x[sl[i].off + j] = out[j];
      }
    }
  }
  if (!kQuant) return;

  if (kTile) {
    float a = vmax[0];
#pragma unroll
    for (int i = 1; i < kStateSlots; ++i) a = fmaxf(a, vmax[i]);
    a = tile8_max(a);
    if ((cq & 7) == 0) tile_max[rw][cq >> 3] = a;
    __syncthreads();
    a = tile_max[0][cq >> 3];
#pragma unroll
    for (int q = 1; q < kStateWaves; ++q) a = fmaxf(a, tile_max[q][cq >> 3]);
    if (rw == 0 && (cq & 7) == 0 && sl[0].nv > 0) absmax[sl[0].blk] = a;
#pragma unroll
    for (int i = 0; i < kStateSlots; ++i) vmax[i] = a;
  } else {
#pragma unroll
    for (int i = 0; i < kStateSlots; ++i) {
      const float a = run32_max(vmax[i]);
      vmax[i] = a;
      if ((cq & 31) == 0 && sl[i].nv > 0) absmax[sl[i].blk] = a;
    }
  }
#pragma unroll
  for (int i = 0; i < kStateSlots; ++i) {
    if (sl[i].nv == 0) continue;
    const double step_rcp = step_reciprocal(vmax[i], levels);
    const float lo = is_unsigned ? 0.0f : -127.0f;
    unsigned c = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) c |= (unsigned(state_code(v[i][j], step_rcp, lo, levels)) & 0xffu) << (8 * j);
    if (vec && sl[i].nv == 4) {
      __builtin_nontemporal_store(c, reinterpret_cast<unsigned*>(codes + sl[i].off));
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j)
        if (j < sl[i].nv) codes[sl[i].off + j] = uint8_t(c >> (8 * j));
    }
  }
}

template <bool kQuant>
__global__ __launch_bounds__(kStateThreads) void state_codec_kernel(
    const TensorDev* __restrict__ T, const Item* __restrict__ items, int64_t item_off,
    int64_t item_count, float* __restrict__ x, uint8_t* __restrict__ codes,
    float* __restrict__ absmax, int is_unsigned, int64_t elem_base, int64_t state_off) {
  __shared__ float tile_max[kStateWaves][kStateCols / 32];
  const int64_t idx = xcd_chunked(blockIdx.x, kXcdChunk);
  if (idx >= item_count) return;
  const Item it = items[item_off + idx];
  const TensorDev t = T[it.tensor];
  if (t.flags & kFlagStateRuns)
    state_codec_item<kQuant, false>(t, it, x, codes, absmax, is_unsigned != 0, elem_base, state_off, tile_max);
  else
    state_codec_item<kQuant, true>(t, it, x, codes, absmax, is_unsigned != 0, elem_base, state_off, tile_max);
}

// -------------------------------------------------------------------------------------------
// launcher (host)
// -------------------------------------------------------------------------------------------
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

int launch_state_codec(bool quantise, const DeviceTables& dev, int64_t item_off, int64_t item_count,
                       float* x, uint8_t* codes, float* absmax, bool is_unsigned, int64_t elem_base,
                       int64_t state_off, hipStream_t st) {
  if (item_count == 0) return RS_OK;
  if (item_count < 0 || item_count > 0x7fffff00LL) return RS_EOVERFLOW;
  const dim3 g{unsigned(xcd_grid(item_count))}, b{unsigned(kStateThreads)};
  if (quantise)
    state_codec_kernel<true><<<g, b, 0, st>>>(dev.tensors, dev.state_items, item_off, item_count, x,
                                              codes, absmax, is_unsigned ? 1 : 0, elem_base, state_off);
  else
    state_codec_kernel<false><<<g, b, 0, st>>>(dev.tensors, dev.state_items, item_off, item_count, x,
                                               codes, absmax, is_unsigned ? 1 : 0, elem_base, state_off);
  return launched();
}

}  // namespace rs
