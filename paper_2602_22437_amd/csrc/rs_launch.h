// Kernel launchers (the .hip files) as seen by the C ABI layer.
#pragma once
#include <hip/hip_runtime_api.h>

#include "rs_internal.h"

namespace rs {

// group-level operators on the bf16 DBuffer; `op` is one of the values below
enum : int { kGroupPack = 0, kGroupUnpack = 1, kGroupPackScaled = 2, kGroupAdd = 3, kGroupScale = 4 };
// rank k's region starts region_stride elements after rank k-1's (S in a plain DBuffer)
int launch_group_op(int op, const DeviceTables& dev, int n, void* const* ptrs, void* dbuf, float alpha,
                    int64_t S, int64_t gpr, int64_t region_stride, int64_t n_payload_gran,
                    int64_t n_padding_gran, hipStream_t st);
int launch_fill_zero(void* dst, int64_t bytes, hipStream_t st);
// ragged_pack for callers that cannot allocate: the pointer table is staged in a fixed array that
// every GPU holds (kScratchTensors pointers), found once per device by scratch_init (the device
// must be current).  host_ptrs[order[j]] is the j-th tensor in the buffer.
constexpr int kScratchTensors = 4096;
int scratch_init(int device);
int launch_pack_staged(const DeviceTables& dev, int n, const void* const* host_ptrs,
                       const int32_t* order, void* dbuf, int64_t S, int64_t gpr,
                       int64_t n_payload_gran, int64_t n_padding_gran, hipStream_t st);
// batch: null, or a device array [partials | out] of batch_count units reduced in one launch
int launch_shard_reduce(const DeviceTables& dev, int n, const void* partials, int64_t row_stride,
                        float* out, int64_t S, int64_t gpr, int rank, int rows, void* const* batch,
                        int batch_count, hipStream_t st);
int launch_block_quant(const DeviceTables& dev, int64_t item_off, int64_t item_count, const void* x,
                       uint8_t* codes, float* scales, void* const* batch, int batch_count,
                       int64_t elem_base, int64_t scale_off, hipStream_t st);
// shard_reduce and block_quant in one pass over the rank's quantisation items; mean_out may be null
int launch_reduce_quant(const DeviceTables& dev, int64_t item_off, int64_t item_count,
                        const void* partials, int64_t row_stride, uint8_t* codes, float* scales,
                        float* mean_out, void* const* batch_in, void* const* batch_out,
                        int batch_count, bool write_means, int64_t elem_base, int64_t scale_off,
                        int world, hipStream_t st);
int launch_dequant_unpack(bool f32_out, const DeviceTables& dev, int n, int64_t n_payload_gran,
                          const uint8_t* codes, const float* scales, void* const* ptrs, int64_t S,
                          int64_t gpr, int64_t region_stride, hipStream_t st);
// fp32 constants of one 8-bit Adam step
struct Adam8Consts {
  float beta1, beta2, one_minus_beta1, one_minus_beta2, eps, step_size, bc2_sqrt, decay;
  double bc2_sqrt_rcp;   // 1 / double(bc2_sqrt), correctly rounded: the divisor every element shares
};
int launch_adam8_step(const DeviceTables& dev, int64_t item_off, int64_t item_count, const float* grad,
                      float* master, void* param_bf16, int8_t* m_codes, uint8_t* v_codes,
                      float* m_absmax, float* v_absmax, void* const* batch, int batch_count,
                      int64_t elem_base, int64_t state_off, const Adam8Consts& c, hipStream_t st);
// the 8-bit codec on its own: fp32 -> codes + absmax (quantise) or back (x is then the output)
int launch_state_codec(bool quantise, const DeviceTables& dev, int64_t item_off, int64_t item_count,
                       float* x, uint8_t* codes, float* absmax, bool is_unsigned, int64_t elem_base,
                       int64_t state_off, hipStream_t st);
int launch_copy_probe(void* dst, const void* src, int64_t bytes, hipStream_t st);

}  // namespace rs
