/*
 * raggedshard.h - C ABI of the MI355X (gfx950) RaggedShard / DBuffer hot path.
 *
 * One FSDP unit's tensors are laid out in a rank-major flat communication buffer
 * ("DBuffer", paper Section 5) by the structure-aware planner (Section 5, problem
 * statement and Algorithm 1) so that every sharding block stays whole on one rank
 * (Section 4, block-wise RaggedShard).  Four HBM-bound kernels move data through it:
 * ragged_pack, shard_reduce, FP8 block_quant and dequant_unpack.
 *
 * Conventions
 *   - All sizes and offsets are in ELEMENTS unless a name says bytes.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP device
 *     memory of the device the plan was uploaded to.  The library never takes
 *     ownership of caller memory.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device
 *     calls enqueue exactly one kernel, never synchronise and never allocate.
 *   - Every function returning int returns RS_OK (0) or a negative RS_E* code and
 *     never aborts; rs_strerror() names the code.
 *   - An uploaded plan and its tables are read-only: any number of threads and streams may
 *     use them at once.  Creating, uploading and destroying an object are for one thread.
 *   - bf16 = 2-byte bfloat16, codes = 1-byte OCP FP8 E4M3 ("fn": bias 7, no inf,
 *     max 448), scales = fp32.
 */
#ifndef RAGGEDSHARD_H
#define RAGGEDSHARD_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  RS_OK = 0,
  RS_EINVAL = -1,        /* bad argument (null, non-positive size, unknown mode, rank out of range) */
  RS_EOVERFLOW = -2,     /* world * S does not fit in 62 bits */
  RS_ENOMEM = -3,        /* host or device allocation failed */
  RS_EALIGN = -4,        /* a device pointer or stride misses its required alignment */
  RS_EUNSUPPORTED = -5,  /* operation undefined for this plan (e.g. FP8 on whole-matrix blocks) */
  RS_EHIP = -6,          /* a HIP runtime call failed (no device, launch error) */
  RS_ENOTUPLOADED = -7,  /* device call before rs_plan_upload */
  RS_ETOOBIG = -8        /* more tensors than the fixed device array of rs_pack_noalloc holds */
};

/* Sharding granularity of one tensor (Section 4: the atomic non-shardable block).
 * Row-wise RaggedShard makes 2-D tiles contiguous: 128 whole rows hold a row of 128x128 tiles
 * (Section 6.4: granularity of 128 rows). */
enum {
  RS_BLOCK_1x128 = 0,    /* 1-D: g = 128 elements; 2-D: g = one row; FP8 blocks are 1x128 runs per row */
  RS_BLOCK_128x128 = 1,  /* 2-D only: g = 128 rows; FP8 blocks are 128x128 tiles, edge tiles partial */
  RS_BLOCK_WHOLE = 2,    /* g = e: the whole tensor on one rank (matrix optimisers, Section 6.3); no FP8 */
  RS_BLOCK_EXPLICIT = 3, /* g = g_explicit elements; no FP8 */
  RS_BLOCK_32x32 = 4     /* 2-D: g = 32 rows; 1-D: g = 128 elements.  The granularity of the block-wise
                            8-bit optimiser state (Section 6.3); no FP8 */
};

/* Tensor orders tried by the planner (Section 5, "heuristic-guided solution": default order,
 * sorted by sharding block size, sorted by tensor shape; the paper adopts the default). */
enum {
  RS_ORDER_DEFAULT = 0,     /* the order of the descriptor array */
  RS_ORDER_BLOCK_SIZE = 1,  /* stable sort by g_t, ascending */
  RS_ORDER_SHAPE = 2,       /* stable sort by (element count, rows, cols), ascending */
  RS_ORDER_BEST = 3,        /* all three; the smallest S wins, the earlier order on ties */
  RS_UNITS_LISTING = 256    /* flag, OR-ed into an order: search only the candidate units of Algorithm
                               1's listing (the running LCM over the ascending distinct block sizes,
                               g_coll first) instead of the wider set rs_plan_create describes */
};

typedef struct rs_tensor_desc {
  int64_t rows;        /* R, or the length n of a 1-D tensor */
  int64_t cols;        /* C; 0 marks a 1-D tensor */
  int32_t block_mode;  /* RS_BLOCK_* */
  int32_t reserved;    /* must be 0 */
  int64_t g_explicit;  /* used by RS_BLOCK_EXPLICIT only */
} rs_tensor_desc;

/* n elements of tensor `tensor`, starting at its element src_off, live at element dst_off
 * of one rank's region [rank*S, (rank+1)*S). */
typedef struct rs_segment {
  int32_t tensor;
  int32_t reserved;
  int64_t src_off;
  int64_t dst_off;
  int64_t n;
} rs_segment;

typedef struct rs_plan rs_plan;                  /* layout plan + device tables, library-owned */
typedef struct rs_tensor_table rs_tensor_table;  /* device copy of n tensor base pointers */
typedef struct rs_shard_batch rs_shard_batch;    /* device copy of the buffers of `count` units' shards */
typedef struct rs_partials_batch rs_partials_batch;  /* the same for the partials and means of `count` units */
typedef struct rs_adam8_batch rs_adam8_batch;    /* the same for the optimiser buffers of `count` units */

int rs_version(void);
const char* rs_strerror(int code);

/* ---- plan (host only; needs no GPU) ------------------------------------------------------
 * Solves  min S  s.t. each tensor is one contiguous interval [l_t, l_t + e_t) of the
 * world*S-element buffer, intervals are disjoint, and every interior rank boundary k*S
 * that falls inside a tensor falls on a multiple of g_t from l_t  (Section 5, the
 * minimisation problem), by Algorithm 1 for the tensor order given: for each candidate unit
 * the smallest feasible multiple is found by bisection with CheckValidShard, which places
 * each tensor at its earliest feasible start; S is the smallest result.  Candidate units, all
 * running LCMs that start from g_coll: over the ascending distinct block sizes (the listing);
 * over the block sizes of the tensors sorted by element count, largest first (the text: the
 * tensors that can contain a whole shard); and every distinct block size on its own.
 *   g_coll = align_bytes / min_itemsize elements (S is a multiple of it, so every rank
 *   region starts align_bytes-aligned for every dtype that shares the plan);
 *   tensor_align_elems = alignment of every l_t, must divide g_coll; 0 selects g_coll.
 * descs: host array of n descriptors, copied.  *out is owned by the library until
 * rs_plan_destroy.  Errors: RS_EINVAL, RS_EOVERFLOW, RS_ENOMEM. */
int rs_plan_create(const rs_tensor_desc* descs, int n, int world, int align_bytes,
                   int min_itemsize, int tensor_align_elems, rs_plan** out);
/* The same with a choice of tensor order (RS_ORDER_*, optionally | RS_UNITS_LISTING for the
 * algorithm exactly as listed).  Tensors keep the caller's indices in every query and pointer
 * table; only their positions in the buffer change. */
int rs_plan_create_ordered(const rs_tensor_desc* descs, int n, int world, int align_bytes,
                           int min_itemsize, int tensor_align_elems, int order, rs_plan** out);
/* The buffer of a group placed RaggedShard(r_t): every block of tensor t on device roots[t]
 * (Section 4: arbitrary sharding distribution; the redistribute target of Algorithm 2, where
 * only the root holds the full matrix).  Device k's region holds the tensors rooted at k in the
 * caller's order, each start a multiple of tensor_align_elems; S is the largest region's extent
 * rounded up to g_coll.  roots: host array of n values in [0, world), else RS_EINVAL.  The plan
 * answers every query and drives every device call like one made by rs_plan_create. */
int rs_plan_create_rooted(const rs_tensor_desc* descs, int n, int world, int align_bytes,
                          int min_itemsize, int tensor_align_elems, const int32_t* roots,
                          rs_plan** out);
void rs_plan_destroy(rs_plan* plan);

/* SelectRoot of Algorithm 2 (distributed Muon, Section 6.3), of which the paper says only that
 * it balances load: longest-processing-time-first.  2-D tensors in descending cost (equal costs in
 * index order) each go to the device with the least accumulated cost, the lowest such device.
 * Cost of an R x C matrix = one quintic Newton-Schulz iteration, a*a*(2b + a) with
 * a = min(R, C), b = max(R, C).  roots (host, n values) receives the device, -1 for 1-D
 * tensors; loads (host, world values, may be NULL) the accumulated cost of every device.
 * block_mode and g_explicit of the descriptors are not used beyond validation. */
int rs_select_roots(const rs_tensor_desc* descs, int n, int world, int32_t* roots, double* loads);

/* Composition with an even Shard(dim > 0) of another placement (Section 4, composing with
 * existing sharding formats): the ragged granularity of the row-major local tensor `shape`
 * (ndim sizes) that never cuts into dimension dim, 0 < dim < ndim:
 * *g_out = lcm(shape[dim] * ... * shape[ndim-1], g_user) elements, for use as g_explicit of an
 * RS_BLOCK_EXPLICIT descriptor.  Errors: RS_EINVAL, RS_EOVERFLOW. */
int rs_shard_dim_granularity(const int64_t* shape, int ndim, int dim, int64_t g_user,
                             int64_t* g_out);

/* CheckValidShard(S) of Algorithm 1 on its own: 1 feasible, 0 infeasible, <0 error.
 * S must be a positive multiple of tensor_align_elems (0 = g_coll). */
int rs_check_valid_shard(const rs_tensor_desc* descs, int n, int world, int align_bytes,
                         int min_itemsize, int tensor_align_elems, int64_t S);

/* Queries (pure).  Output arrays are caller-owned host memory. */
int rs_plan_num_tensors(const rs_plan* plan);
int rs_plan_world(const rs_plan* plan);
int64_t rs_plan_shard_elems(const rs_plan* plan);    /* S */
int64_t rs_plan_total_elems(const rs_plan* plan);    /* world * S */
int64_t rs_plan_payload_elems(const rs_plan* plan);  /* sum of e_t */
int64_t rs_plan_padding_elems(const rs_plan* plan);  /* world * S - payload */
int64_t rs_plan_num_scales(const rs_plan* plan);     /* FP8 blocks of the whole unit */
/* Buffer order: out[j] = index of the j-th tensor in the buffer; cap must be >= n. */
int rs_plan_order(const rs_plan* plan, int32_t* out, int cap);
/* l_t for every tensor; cap must be >= n. */
int rs_plan_offsets(const rs_plan* plan, int64_t* out, int cap);
/* first scale index of every tensor plus the total (n + 1 values; cap >= n + 1).  Scales form
 * one flat fp32 array in buffer order: tensor-major, then block row, then block column. */
int rs_plan_scale_bases(const rs_plan* plan, int64_t* out, int cap);
/* [lo, hi): the scales rank owns; contiguous because blocks are whole on a rank. */
int rs_plan_scale_range(const rs_plan* plan, int rank, int64_t* lo, int64_t* hi);
/* Writes up to cap segments of the rank and returns how many the rank has (may exceed cap). */
int rs_plan_rank_segments(const rs_plan* plan, int rank, rs_segment* out, int cap);

/* ---- device set-up -------------------------------------------------------------------------
 * Builds the plan's device tables on HIP device `device` (hipMalloc + copy, synchronous).
 * Call once before any device call; freed by rs_plan_destroy.  RS_EHIP without a GPU. */
int rs_plan_upload(rs_plan* plan, int device);

/* The DBuffer's persistent tensor -> address mapping (Section 5): uploads n device base
 * pointers (host array `ptrs`, one per tensor, each tensor contiguous row-major) to the
 * plan's device.  The table may be reused by any number of calls. */
int rs_tensor_table_create(const rs_plan* plan, const void* const* ptrs, rs_tensor_table** out);
void rs_tensor_table_destroy(rs_tensor_table* table);

/* ---- ragged_pack: the fused group copy + zero of the DBuffer (Section 5) ---------------------
 * dbuf[l_t + i] = src_t[i] for every tensor, every other element of dbuf[0, world*S) = +0.
 * src: table of bf16 device tensors; dbuf: device, world*S bf16, 16-byte aligned (RS_EALIGN). */
int rs_pack(const rs_plan* plan, const rs_tensor_table* src, void* dbuf, void* stream);

/* rs_pack for callers that cannot allocate device memory: code under HIP graph capture, tight
 * serving loops, harnesses that forbid hipMalloc, and callers whose source tensors move from call
 * to call, for whom a table from rs_tensor_table_create would have to be made (and freed) every
 * time.  Same result as rs_pack, bit for bit.  src_ptrs: HOST array of n device pointers (bf16
 * tensors, element-aligned, none null), read before the call returns.  The pointers travel as
 * kernel arguments into a fixed array of RS_NOALLOC_MAX_TENSORS pointers (32 KiB) that every GPU
 * the library runs on holds until the process ends; the call enqueues ceil(n / 256) small staging
 * kernels and the copy kernel on `stream` and calls no allocating routine.
 * n > RS_NOALLOC_MAX_TENSORS: RS_ETOOBIG.  Every call on a GPU shares that GPU's array: calls that
 * may overlap in time on one GPU (different streams or threads) race; calls on one stream are safe. */
#define RS_NOALLOC_MAX_TENSORS 4096
int rs_pack_noalloc(const rs_plan* plan, const void* const* src_ptrs, void* dbuf, void* stream);

/* Inverse group copy: dst_t[i] = dbuf[l_t + i] (bf16 DBuffer -> per-tensor bf16). */
int rs_unpack_bf16(const rs_plan* plan, const void* dbuf, const rs_tensor_table* dst, void* stream);

/* ---- regions gathered over a 2-D device mesh (Section 4: RaggedShard composed with the Shard(0)
 * of expert or tensor parallelism; the stride metadata of StridedRaggedShard) ---------------------
 * The same two copies on a buffer in which rank k's region starts at element k * region_stride
 * instead of k * S.  When a parameter is first split over G devices of the other mesh dimension
 * and each part is ragged-sharded over `world` devices, the buffer gathered over the whole mesh
 * holds the regions device-major (FSDP rank outermost): part g's regions are read with
 * dbuf + g * S and region_stride = G * S, and a tensor table over the g-th slices of the full
 * tensors - G launches materialise the full tensors, no intermediate copy.
 * region_stride >= S (RS_EINVAL), a multiple of 8 elements (RS_EALIGN); rs_pack_strided zeroes
 * the padding of the regions it addresses and touches nothing between them. */
int rs_pack_strided(const rs_plan* plan, const rs_tensor_table* src, void* dbuf, int64_t region_stride,
                    void* stream);
int rs_unpack_bf16_strided(const rs_plan* plan, const void* dbuf, int64_t region_stride,
                           const rs_tensor_table* dst, void* stream);

/* ---- the other group-level operators of the DBuffer (Section 5: the add, scale, zero and copy
 * kernels that each tensor would launch around a collective, fused across the group) ----------
 * alpha is an fp32 factor (finite, else RS_EINVAL); every product and sum is one fp32
 * operation in the order written and the result is rounded to bf16 once, to nearest even.
 * dbuf: device, world*S bf16, 16-byte aligned; src: table of bf16 device tensors.
 *   rs_pack_scaled  dbuf[l_t + i] = bf16(src_t[i] * alpha), padding = +0  (copy-in + pre-division)
 *   rs_group_add    dbuf[l_t + i] = bf16(dbuf[l_t + i] + alpha * src_t[i]) (gradient accumulation)
 *   rs_group_scale  dbuf[l_t + i] = bf16(dbuf[l_t + i] * alpha)
 *   rs_group_zero   dbuf[0, world*S) = +0
 * rs_group_add and rs_group_scale leave padding as it is. */
int rs_pack_scaled(const rs_plan* plan, const rs_tensor_table* src, float alpha, void* dbuf,
                   void* stream);
int rs_group_add(const rs_plan* plan, const rs_tensor_table* src, float alpha, void* dbuf,
                 void* stream);
int rs_group_scale(const rs_plan* plan, float alpha, void* dbuf, void* stream);
int rs_group_zero(const rs_plan* plan, void* dbuf, void* stream);

/* ---- shard_reduce: the arithmetic of the gradient ReduceScatter as one rank sees it --------
 * (Section 2.3).  out[i] = (1/world) * sum_w partials[w*row_stride + i] for i in the
 * payload of rank's region, 0 on its padding; fp32 accumulation in a fixed order, so the result
 * is reproducible bit for bit: partial w is added, in increasing w, to running sum (w mod 8);
 * the eight sums combine as ((a0+a1)+(a2+a3))+((a4+a5)+(a6+a7)); then one multiply by fp32(1/world).
 * partials: device, `world` rows of S bf16, row_stride elements apart (multiple of 8,
 * base 16-byte aligned); out: device, S fp32, 16-byte aligned. */
int rs_reduce(const rs_plan* plan, int rank, const void* partials, int64_t row_stride,
              float* out, void* stream);
/* The same mean over `rows` partials (1 <= rows <= 2^24) instead of `world`: the arithmetic one rank
 * performs in the 2-D gradient reduction of an N-D DBuffer (Section 5: ReduceScatter along one
 * mesh dimension, AllReduce along the other), where a region receives world * replicas
 * contributions, or one per replica in the second step.  rs_reduce is rows == world. */
int rs_reduce_rows(const rs_plan* plan, int rank, const void* partials, int rows, int64_t row_stride,
                   float* out, void* stream);

/* The same mean for rank `rank`'s region of `count` units that share this plan (the layers of a
 * model) in one launch, as the DBuffer fuses identical kernels across a group (Section 5): the
 * region of one unit may be too short to fill the GPU.  partials / outs: host arrays of `count`
 * device pointers with rs_reduce's meaning and alignment, all with the one row_stride; uploaded
 * once, reusable by any number of calls.  count <= 65535.  Bit for bit the result of rs_reduce on
 * every unit (same summation order). */
int rs_partials_batch_create(const rs_plan* plan, int rank, int count, const void* const* partials,
                             int64_t row_stride, float* const* outs, rs_partials_batch** out);
void rs_partials_batch_destroy(rs_partials_batch* batch);
int rs_reduce_batch(const rs_plan* plan, const rs_partials_batch* batch, void* stream);

/* ---- block_quant: communication-free block-wise FP8 of the local shard (Sections 2.1, 4) ----
 * Per block: amax = max|x|, scale = amax/448 (fp32), code = E4M3 RNE of clamp(x/scale, +-448);
 * an all-zero block gives scale 0 and codes 0x00.  Padding codes are 0x00.
 * rank >= 0: shard/codes point at that rank's region (S elements), scales at its slice
 * [lo, hi) of the scale array.  rank == -1: all ranks at once (world*S elements, all scales).
 * shard: device bf16, codes: device uint8, both 16-byte aligned.  RS_EUNSUPPORTED if the plan
 * holds a tensor without FP8 blocks. */
int rs_quantize(const rs_plan* plan, int rank, const void* shard, uint8_t* codes, float* scales,
                void* stream);

/* The same operation for rank `rank`'s shard of `count` units that share this plan (the
 * transformer layers of a model), fused into one launch as the DBuffer fuses identical
 * kernels across a group (Section 5): one shard of one unit is too small to fill the GPU.
 * shards / codes / scales: host arrays of `count` device pointers with rs_quantize's meaning
 * and alignment for that rank; they are uploaded once and may be reused by any number of calls.
 * count <= 65535.  rs_quantize_batch == rs_quantize(plan, rank, shards[u], codes[u], scales[u])
 * for every u, bit for bit. */
int rs_shard_batch_create(const rs_plan* plan, int rank, int count, const void* const* shards,
                          uint8_t* const* codes, float* const* scales, rs_shard_batch** out);
void rs_shard_batch_destroy(rs_shard_batch* batch);
int rs_quantize_batch(const rs_plan* plan, const rs_shard_batch* batch, void* stream);

/* ---- shard_reduce and block_quant fused: the mean of the partials leaves the chip as FP8 ----
 * A group-level fusion in the sense of Section 5: where the mean itself is what travels next
 * (quantised gradient exchange between replicas), it is formed in registers and written as codes
 * and scales only, which saves writing and re-reading S fp32 values.
 *   mean[i] = rs_reduce's out[i], bit for bit (same summation order);
 *   per block: amax = max|mean|, scale = amax/448 (fp32), code = E4M3 RNE of
 *   clamp(mean/scale, +-448) with a correctly rounded fp32 division; a block whose scale is 0
 *   (all zero, or amax so small that amax/448 rounds to 0 in fp32, which needs amax below 2^-140)
 *   gives scale 0 and codes 0x00.  Padding codes are 0x00.
 * The fp32 mean is quantised as it is, with no rounding to bf16 in between: the codes are in
 * general NOT those of rs_reduce -> bf16 -> rs_quantize, which rounds twice.
 * partials, row_stride: as for rs_reduce.  codes: device, S uint8, 16-byte aligned; scales:
 * device, the rank's slice [lo, hi).  mean_out: NULL, or device S fp32, 16-byte aligned, which
 * then also receives the mean (0 on padding).  RS_EUNSUPPORTED if the plan holds a tensor
 * without FP8 blocks. */
int rs_reduce_quantize(const rs_plan* plan, int rank, const void* partials, int64_t row_stride,
                       uint8_t* codes, float* scales, float* mean_out, void* stream);

/* The same for rank `rank`'s region of `count` units that share this plan, in one launch (the
 * group-level fusion of Section 5 again: a unit's shard holds too few blocks to occupy the GPU).
 * in: the units' partial buffers and row stride (rs_partials_batch_create); out: their code and
 * scale buffers (rs_shard_batch_create; its shard pointers are not read).  Both must have been
 * made for this plan with the same rank and count, else RS_EINVAL.  write_means != 0: the fp32
 * mean of unit u is also written to the partials batch's outs[u] (0 on padding); otherwise
 * those buffers are left alone.  Equal to rs_reduce_quantize on every unit, bit for bit. */
int rs_reduce_quantize_batch(const rs_plan* plan, const rs_partials_batch* in,
                             const rs_shard_batch* out, int write_means, void* stream);

/* ---- dequant_unpack: gathered FP8 unit -> per-parameter bf16 --------------------------------
 * dst_t[i] = bf16_rne( value(codes[l_t + i]) * scales[block of i] ).
 * codes: device, world*S uint8, 16-byte aligned; scales: device, all of the unit's scales. */
int rs_unpack(const rs_plan* plan, const uint8_t* codes, const float* scales,
              const rs_tensor_table* dst, void* stream);

/* The same into fp32 tensors (the fp32 master copy of the gathered parameters, without the
 * detour through bf16): dst_t[i] = value(codes[l_t + i]) * scales[block of i], one fp32 multiply.
 * dst: table of fp32 device tensors (4-byte aligned, else RS_EALIGN). */
int rs_unpack_f32(const rs_plan* plan, const uint8_t* codes, const float* scales,
                  const rs_tensor_table* dst, void* stream);

/* The same two on a code buffer gathered over a 2-D device mesh (Section 4, the stride metadata of
 * StridedRaggedShard; see rs_unpack_bf16_strided): rank k's S code bytes start at byte
 * k * region_stride.  With the parameter split over G devices of the other mesh dimension, part g is
 * read with codes + g * S, region_stride = G * S, the scale array of part g (every part has its own,
 * in the plan's order) and a tensor table over the g-th slices of the full tensors.
 * region_stride >= S (RS_EINVAL), a multiple of 8 (RS_EALIGN). */
int rs_unpack_strided(const rs_plan* plan, const uint8_t* codes, int64_t region_stride,
                      const float* scales, const rs_tensor_table* dst, void* stream);
int rs_unpack_f32_strided(const rs_plan* plan, const uint8_t* codes, int64_t region_stride,
                          const float* scales, const rs_tensor_table* dst, void* stream);

/* ---- block-wise 8-bit optimiser state on the local shard (Section 6.3, "8-bit Adam") ---------
 * The two Adam moments of rank's shard are held as 8-bit codes in blocks that never cross a
 * rank boundary, so a rank updates and re-quantises its state with no communication.
 * State blocks are the finest blocks that are whole on a rank: 32x32 tiles (edge tiles partial)
 * of a 2-D tensor in RS_BLOCK_32x32 or RS_BLOCK_128x128 mode; runs of 128 along each row (the
 * last run of a row short) of a 2-D tensor in RS_BLOCK_1x128 mode; runs of 128 elements of a
 * 1-D tensor in RS_BLOCK_32x32 or RS_BLOCK_1x128 mode.  A plan holding any other tensor has no
 * 8-bit state: RS_EUNSUPPORTED.  Blocks are numbered
 * like FP8 scales: tensor-major in buffer order, block row, block column; a rank owns a
 * contiguous range.  Codes: first moment m, int8, step a/127 (a = the block's max |m|),
 * code = rint(m / step); second moment v >= 0, uint8, step a/255; all-zero block: a = 0,
 * codes 0.  All-zero codes and absmax are the valid initial state. */
int64_t rs_plan_num_state_blocks(const rs_plan* plan);   /* whole unit; RS_EUNSUPPORTED if undefined */
/* first state block of every tensor plus the total (n + 1 values; cap >= n + 1) */
int rs_plan_state_bases(const rs_plan* plan, int64_t* out, int cap);
int rs_plan_state_range(const rs_plan* plan, int rank, int64_t* lo, int64_t* hi);

/* The codec on its own over rank's shard, one launch each (state initialised from, or exported to,
 * fp32 moments).  is_unsigned = 0: the first-moment map (int8, step a/127, a = max |x| of the
 * block); 1: the second-moment map (uint8, step a/255, a = max x, inputs >= 0).
 *   rs_state_quantize    codes = rint(src / step), absmax = a per block  (all-zero block: 0, codes 0)
 *   rs_state_dequantize  dst = code * (absmax / levels), one fp32 division per block, one multiply
 * src / dst: device fp32, S elements at the region's element offsets; codes: device, S bytes;
 * absmax: device fp32, the rank's slice of the block array.  Bases 16-byte aligned (absmax: 4).
 * Padding positions are neither read nor written. */
int rs_state_quantize(const rs_plan* plan, int rank, const float* src, int is_unsigned, void* codes,
                      float* absmax, void* stream);
int rs_state_dequantize(const rs_plan* plan, int rank, const void* codes, const float* absmax,
                        int is_unsigned, float* dst, void* stream);

typedef struct rs_adam8_hyper {
  double lr, beta1, beta2, eps, weight_decay;
  int64_t step;        /* 1 for the first update */
} rs_adam8_hyper;

/* One AdamW step on rank's shard, one launch.  Per payload element, in fp32, every operation
 * rounded on its own in this order:
 *   m_old = code_m * (a_m / 127);   v_old = code_v * (a_v / 255)
 *   m = beta1 * m_old + (1 - beta1) * g;      v = beta2 * v_old + (1 - beta2) * (g * g)
 *   w = w * (1 - lr * weight_decay)
 *   w = w - (lr / bc1) * (m / (sqrt(v) / sqrt(bc2) + eps)),     bc_i = 1 - beta_i^step
 *   param = bf16(w) (nearest even)
 * then m and v are quantised again per block.  The constants beta_i, (1 - beta_i), eps, lr / bc1,
 * sqrt(bc2), (1 - lr * weight_decay) are evaluated in double precision and rounded once to fp32.
 * grad (in), master (in/out): device fp32, S elements at the region's element offsets;
 * param_bf16 (out, may be NULL): device bf16, S elements; m_codes / v_codes (in/out): device,
 * S bytes each; m_absmax / v_absmax (in/out): device fp32, the rank's slice [lo, hi) of the
 * state-block arrays.  Array bases 16-byte aligned (absmax: 4).  Padding positions of every
 * array are neither read nor written.  RS_EINVAL unless lr, weight_decay finite, 0 <= beta_i < 1,
 * eps > 0, step >= 1. */
int rs_adam8_step(const rs_plan* plan, int rank, const rs_adam8_hyper* hyper, const float* grad,
                  float* master, void* param_bf16, int8_t* m_codes, uint8_t* v_codes,
                  float* m_absmax, float* v_absmax, void* stream);

/* The same step for rank's shard of `count` units that share this plan (the layers of a model)
 * in one launch, as an optimiser applies one update to all parameters: one unit's shard is too
 * small to fill the GPU.  Each argument is a host array of `count` device pointers with
 * rs_adam8_step's meaning and alignment (params_bf16 may be NULL, or hold NULL entries); they
 * are uploaded once and may be reused by any number of steps.  count <= 65535.  Bit for bit the
 * result of rs_adam8_step on every unit. */
int rs_adam8_batch_create(const rs_plan* plan, int rank, int count, const float* const* grads,
                          float* const* masters, void* const* params_bf16, int8_t* const* m_codes,
                          uint8_t* const* v_codes, float* const* m_absmax, float* const* v_absmax,
                          rs_adam8_batch** out);
void rs_adam8_batch_destroy(rs_adam8_batch* batch);
int rs_adam8_step_batch(const rs_plan* plan, const rs_adam8_batch* batch, const rs_adam8_hyper* hyper,
                        void* stream);

/* ---- bandwidth probe: plain 16-byte-vector device copy of `bytes` (multiple of 16) ---------
 * Not part of the method: the measured ceiling the four kernels are held against, and the
 * known-size launch that calibrates HBM byte counters. */
int rs_copy_probe(void* dst, const void* src, int64_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* RAGGEDSHARD_H */
