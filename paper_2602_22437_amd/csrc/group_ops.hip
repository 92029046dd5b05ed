// Group-level operators of the DBuffer and the plain-copy probe (gfx950, wave64).
//
// Common shape of the streaming kernels: one 16-byte vector per lane per access and a very large
// grid (a plain copy on MI355X is fastest that way: no grid-stride loop, no multi-vector tiles),
// single-wavefront workgroups for copies (measured 3-4 % faster than 256 lanes), non-temporal
// loads/stores since nothing is reused, and one 8-byte table read per workgroup to find its
// granule and its tensor.  No MFMA: nothing here is a contraction.
#include <mutex>

#include "device_util.h"

namespace rs {

// -------------------------------------------------------------------------------------------
// Group-level operators of the DBuffer: one launch for all tensors of the unit.
//   pack (copy + zero), its inverse, pack with a scale factor, accumulate (axpy), scale.
// Four single-wavefront workgroups per granule (kGranule buffer elements of one rank region)
// that holds payload; the two pack forms add one workgroup per pure-padding granule to zero it,
// the others never touch padding.  fp32 arithmetic, one rounding to bf16 (nearest even).
// -------------------------------------------------------------------------------------------
constexpr int kCopyThreads = 64;
constexpr int kCopyParts = kGranule / (kCopyThreads * 8);  // workgroups per granule: 4

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
    const TensorDev* __restrict__ T, int n, const GranRef* __restrict__ granules,
    const int32_t* __restrict__ padding,
    unsigned n_copy_groups, void* const* __restrict__ ptrs, uint16_t* __restrict__ dbuf, int64_t S,
    int64_t gpr, int64_t region_stride, float alpha) {
  constexpr bool kFillsPadding = kOp == kGroupPack || kOp == kGroupPackScaled;
  constexpr bool kReadsBuffer = kOp == kGroupUnpack || kOp == kGroupAdd || kOp == kGroupScale;
  constexpr bool kUsesTensors = kOp != kGroupScale;
  if (kFillsPadding && blockIdx.x >= n_copy_groups) {
    // a granule of nothing but padding: this wavefront zeroes all of it
    const unsigned gid = unsigned(padding[blockIdx.x - n_copy_groups]);
    const unsigned k = gid / unsigned(gpr);
    const int64_t i0 = int64_t(gid - k * unsigned(gpr)) * kGranule;
    const int len = int(min(int64_t(kGranule), S - i0));
#pragma unroll
    for (int h = 0; h < kCopyParts; ++h) {
      const int lo = (h * kCopyThreads + int(threadIdx.x)) * 8;
      if (lo < len) st16(dbuf + k * region_stride + i0 + lo, u32x4{0, 0, 0, 0});
    }
    return;
  }
  const unsigned slot = blockIdx.x / kCopyParts, part = blockIdx.x % kCopyParts;
  // one 8-byte read: the granule and its first tensor (a payload granule: t0 < n and tensor t0
  // starts before the granule ends)
  const long long packed = reinterpret_cast<const long long*>(granules)[slot];
  const int t0 = int32_t(packed >> 32);
  // Everything the common case needs is requested at once, ahead of the index arithmetic (one
  // round of table reads, one branch): the tensor's interval and its base pointer.
  const int64_t ell = T[t0].ell, end = ell + T[t0].e;
  uint16_t* const tensor = kUsesTensors ? reinterpret_cast<uint16_t*>(ptrs[t0]) : nullptr;
  const unsigned bid = unsigned(packed);             // granule ids and gpr fit 31 bits
  const unsigned k = bid / unsigned(gpr);
  const int64_t i0 = int64_t(bid - k * unsigned(gpr)) * kGranule;
  const int64_t d0 = k * S + i0;
  const int len = int(min(int64_t(kGranule), S - i0));
  const int lane_off = (int(part) * kCopyThreads + int(threadIdx.x)) * 8;
  if (lane_off >= len) return;
  const int64_t d = d0 + lane_off;          // logical buffer position: what the tables speak of
  // where it lives: rank regions are region_stride elements apart (S in a plain DBuffer)
  uint16_t* const at = dbuf + k * region_stride + i0 + lane_off;
  uint16_t* const base = kUsesTensors ? tensor + (d0 - ell) : nullptr;
  const bool inside = (ell <= d0) & (d0 + len <= end);
  const bool usable = !kUsesTensors | ((reinterpret_cast<uintptr_t>(base) & 15) == 0);
  if (inside & usable) {
    // the whole granule lies inside tensor t0 (the common case by far)
    if (kOp == kGroupScale)
      st16(at, scale8(ld16(at), alpha));
    else if (kOp == kGroupUnpack)
      st16(base + lane_off, ld16(at));
    else if (kOp == kGroupPack)
      st16(at, ld16(base + lane_off));
    else if (kOp == kGroupPackScaled)
      st16(at, scale8(ld16(base + lane_off), alpha));
    else
      st16(at, axpy8(ld16(at), ld16(base + lane_off), alpha));
    return;
  }

  // Mixed granule (tensor boundaries, padding, or a source that is not 16-byte aligned):
  // resolve every element on its own.
  int s = t0;
  uint16_t vals[8] = {0, 0, 0, 0, 0, 0, 0, 0};
  if (kReadsBuffer) {
    const u32x4 v = ld16(at);
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
    st16(at, v);
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
// plain copy: the measured ceiling and the counter calibration launch
// -------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kCopyThreads) void copy_probe_kernel(const u32x4* __restrict__ src,
                                                                 u32x4* __restrict__ dst,
                                                                 int64_t nvec) {
  const int64_t i = int64_t(blockIdx.x) * kCopyThreads + threadIdx.x;
  if (i < nvec) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

// -------------------------------------------------------------------------------------------
// Pointer staging for callers that cannot allocate: the tensor -> address table of one call lives
// in a fixed array in device memory instead of a table made by hipMalloc.  The host hands the
// pointers over as kernel arguments (kStageChunk per launch), so nothing is copied from host
// memory either.  One array per GPU, shared by every call on that GPU.
// -------------------------------------------------------------------------------------------
static_assert(kScratchTensors == RS_NOALLOC_MAX_TENSORS, "the header states the array's capacity");
static __device__ __align__(256) unsigned char scratch[kScratchTensors * sizeof(void*)];

constexpr int kStageChunk = 256;           // 2 KiB of kernel arguments
struct PtrChunk {
  void* p[kStageChunk];
};

__global__ __launch_bounds__(kStageChunk) void stage_ptrs_kernel(PtrChunk chunk, void** table,
                                                                int first, int count) {
  const int i = threadIdx.x;
  if (i < count) table[first + i] = chunk.p[i];
}

namespace {
constexpr int kMaxDevices = 64;
std::mutex scratch_mutex;
void* scratch_addr[kMaxDevices] = {};      // device address of `scratch` on every GPU seen so far
}  // namespace

// Looks up where `scratch` lives on `device`, which must be the current device.  The array's name
// is only a host-side handle: kernels and copies get the address found here.
int scratch_init(int device) {
  if (device < 0 || device >= kMaxDevices) return RS_EINVAL;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (scratch_addr[device]) return RS_OK;
  void* addr = nullptr;
  if (hipGetSymbolAddress(&addr, HIP_SYMBOL(scratch)) != hipSuccess || !addr) return RS_EHIP;
  scratch_addr[device] = addr;
  return RS_OK;
}

static void* scratch_of(int device) {
  if (device < 0 || device >= kMaxDevices) return nullptr;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  return scratch_addr[device];
}

// -------------------------------------------------------------------------------------------
// launchers (host)
// -------------------------------------------------------------------------------------------
int launch_group_op(int op, const DeviceTables& dev, int n, void* const* ptrs, void* dbuf, float alpha,
                    int64_t S, int64_t gpr, int64_t region_stride, int64_t n_payload_gran,
                    int64_t n_padding_gran, hipStream_t st) {
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
  group_op_kernel<OP><<<g, b, 0, st>>>(dev.tensors, n, dev.payload_gran, dev.padding_gran,     \
                                       unsigned(copy_groups), ptrs, db, S, gpr, region_stride, \
                                       alpha)
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

// ragged_pack with the pointer table staged in the GPU's fixed array: host_ptrs[order[j]] is the
// j-th tensor in the buffer.  Launches ceil(n / kStageChunk) staging kernels and the copy kernel
// on `st`; allocates nothing.
int launch_pack_staged(const DeviceTables& dev, int n, const void* const* host_ptrs,
                       const int32_t* order, void* dbuf, int64_t S, int64_t gpr,
                       int64_t n_payload_gran, int64_t n_padding_gran, hipStream_t st) {
  if (n > kScratchTensors) return RS_ETOOBIG;
  int rc = scratch_init(dev.device);
  if (rc != RS_OK) return rc;
  void** table = static_cast<void**>(scratch_of(dev.device));
  if (!table) return RS_EHIP;
  for (int first = 0; first < n; first += kStageChunk) {
    const int count = n - first < kStageChunk ? n - first : kStageChunk;
    PtrChunk chunk;
    for (int i = 0; i < count; ++i) chunk.p[i] = const_cast<void*>(host_ptrs[order[first + i]]);
    for (int i = count; i < kStageChunk; ++i) chunk.p[i] = nullptr;
    stage_ptrs_kernel<<<dim3(1), dim3(kStageChunk), 0, st>>>(chunk, table, first, count);
    rc = launched();
    if (rc != RS_OK) return rc;
  }
  return launch_group_op(kGroupPack, dev, n, table, dbuf, 1.0f, S, gpr,
                         S, n_payload_gran, n_padding_gran, st);
}

int launch_fill_zero(void* dst, int64_t bytes, hipStream_t st) {
  const int64_t nvec = bytes / 16;
  const int64_t grid = (nvec + kFillThreads - 1) / kFillThreads;
  if (grid == 0) return RS_OK;
  if (grid > 0x7fffffffLL) return RS_EOVERFLOW;
  fill_zero_kernel<<<dim3(unsigned(grid)), dim3(kFillThreads), 0, st>>>(static_cast<u32x4*>(dst), nvec);
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
