// C ABI of the library: argument checking, plan objects, device tables, kernel launches.
#include <hip/hip_runtime_api.h>

#include <cmath>
#include <cstring>
#include <memory>
#include <new>

#include "raggedshard.h"
#include "rs_internal.h"
#include "rs_launch.h"

namespace {

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

// Device calls require the plan's device to be the caller's current one.
int check_device(const rs_plan* plan) {
  if (!plan) return RS_EINVAL;
  if (plan->dev.device < 0) return RS_ENOTUPLOADED;
  int cur = -1;
  if (hipGetDevice(&cur) != hipSuccess) return RS_EHIP;
  return cur == plan->dev.device ? RS_OK : RS_EINVAL;
}

int check_table(const rs_plan* plan, const rs_tensor_table* tab) {
  if (!tab || !tab->ptrs) return RS_EINVAL;
  if (tab->owner != plan || tab->n != int(plan->t.size())) return RS_EINVAL;
  return RS_OK;
}

template <typename T>
int upload(const std::vector<T>& host, T** dev) {
  *dev = nullptr;
  if (host.empty()) return RS_OK;
  const size_t bytes = host.size() * sizeof(T);
  if (hipMalloc(reinterpret_cast<void**>(dev), bytes) != hipSuccess) return RS_ENOMEM;
  if (hipMemcpy(*dev, host.data(), bytes, hipMemcpyHostToDevice) != hipSuccess) return RS_EHIP;
  return RS_OK;
}

void free_device_tables(rs::DeviceTables* d) {
  if (d->device < 0) return;
  int cur = -1;
  const bool have = hipGetDevice(&cur) == hipSuccess;
  if (have && cur != d->device) (void)hipSetDevice(d->device);
  if (d->tensors) (void)hipFree(d->tensors);
  if (d->gran_first) (void)hipFree(d->gran_first);
  if (d->items) (void)hipFree(d->items);
  if (d->payload_gran) (void)hipFree(d->payload_gran);
  if (d->padding_gran) (void)hipFree(d->padding_gran);
  if (d->state_items) (void)hipFree(d->state_items);
  if (have && cur != d->device) (void)hipSetDevice(cur);
  *d = rs::DeviceTables{};
}

// Number of scales in front of buffer position x: the blocks of all whole granules (a row of
// tiles, a row of 1x128 runs, or one 1-D run) that start before x.
int64_t scales_in_front(const rs_plan& plan, int64_t x) {
  int64_t cnt = 0;
  for (const rs::TensorHost& h : plan.t) {
    if (!h.quant || x <= h.ell) continue;
    int64_t granules = (x - h.ell + h.g - 1) / h.g;
    if (granules > h.u) granules = h.u;
    cnt += granules * (h.cols > 0 ? h.nbc : 1);
  }
  return cnt;
}

// Number of optimiser-state blocks in front of buffer position x (a rank boundary: it falls
// between rows of state tiles, or between runs of 128).
int64_t state_blocks_in_front(const rs_plan& plan, int64_t x) {
  int64_t cnt = 0;
  for (const rs::TensorHost& h : plan.t) {
    if (!h.state || x <= h.ell) continue;
    const int64_t have = x - h.ell < h.e ? x - h.ell : h.e;
    if (h.cols == 0)
      cnt += (have + 127) / 128;
    else if (h.state_runs)
      cnt += have / h.cols * h.sbc;
    else
      cnt += (have / h.cols + 31) / 32 * h.sbc;
  }
  return cnt;
}

// Host staging array for a device pointer table; empty when the allocation fails.
struct Staging {
  explicit Staging(size_t n) : count(n), data(new (std::nothrow) void*[n]()) {}
  size_t size() const { return count; }
  void*& operator[](size_t i) { return data[i]; }
  size_t count;
  std::unique_ptr<void*[]> data;
};

int build_plan(const rs_tensor_desc* descs, int n, int world, int align_bytes, int min_itemsize,
               int tensor_align_elems, std::vector<rs::TensorHost>* t, int64_t* g_coll, int64_t* A) {
  if (!descs || n <= 0 || world <= 0 || align_bytes <= 0 || min_itemsize <= 0 ||
      tensor_align_elems < 0)
    return RS_EINVAL;
  if (align_bytes % min_itemsize != 0) return RS_EINVAL;
  *g_coll = align_bytes / min_itemsize;
  *A = tensor_align_elems == 0 ? *g_coll : tensor_align_elems;
  if (*g_coll % *A != 0) return RS_EINVAL;
  return rs::describe_tensors(descs, n, t);
}

// Fills in what follows from the starts (given in buffer order): scale and state-block numbering
// and the per-rank ranges of both.
void finish_plan(rs_plan* p, const std::vector<int64_t>& starts) {
  int64_t sb = 0, stb = 0;
  p->all_quant = true;
  p->all_state = true;
  for (size_t i = 0; i < p->t.size(); ++i) {
    p->t[i].ell = starts[i];
    p->t[i].scale_base = sb;
    sb += p->t[i].nbr * p->t[i].nbc;
    p->t[i].state_base = stb;
    stb += p->t[i].sbr * p->t[i].sbc;
    p->payload += p->t[i].e;
    p->all_quant = p->all_quant && p->t[i].quant;
    p->all_state = p->all_state && p->t[i].state;
  }
  p->num_scales = sb;
  p->num_state_blocks = stb;
  p->scale_begin.resize(size_t(p->world) + 1);
  p->state_begin.assign(size_t(p->world) + 1, 0);
  for (int64_t k = 0; k <= p->world; ++k) {
    p->scale_begin[size_t(k)] = scales_in_front(*p, k * p->S);
    if (p->all_state) p->state_begin[size_t(k)] = state_blocks_in_front(*p, k * p->S);
  }
}

}  // namespace

extern "C" {

int rs_version(void) { return 170; }

const char* rs_strerror(int code) {
  switch (code) {
    case RS_OK: return "ok";
    case RS_EINVAL: return "invalid argument";
    case RS_EOVERFLOW: return "size overflow";
    case RS_ENOMEM: return "out of memory";
    case RS_EALIGN: return "pointer or stride not aligned";
    case RS_EUNSUPPORTED: return "operation not supported for this plan";
    case RS_EHIP: return "HIP runtime error";
    case RS_ENOTUPLOADED: return "plan tables not uploaded to a device";
    case RS_ETOOBIG: return "more tensors than the fixed device array of rs_pack_noalloc holds";
    default: return "unknown error";
  }
}

int rs_plan_create_ordered(const rs_tensor_desc* descs, int n, int world, int align_bytes,
                           int min_itemsize, int tensor_align_elems, int order, rs_plan** out) {
  if (!out) return RS_EINVAL;
  *out = nullptr;
  const bool listing_only = (order & RS_UNITS_LISTING) != 0;
  order &= ~RS_UNITS_LISTING;
  if (order < RS_ORDER_DEFAULT || order > RS_ORDER_BEST) return RS_EINVAL;
  try {
    std::vector<rs::TensorHost> listed;
    int64_t g_coll = 0, A = 0;
    int rc = build_plan(descs, n, world, align_bytes, min_itemsize, tensor_align_elems, &listed,
                        &g_coll, &A);
    if (rc != RS_OK) return rc;

    // the candidate orders, in the heuristic's sequence; a later one must be strictly better
    std::vector<int> orders;
    if (order == RS_ORDER_BEST)
      orders = {RS_ORDER_DEFAULT, RS_ORDER_BLOCK_SIZE, RS_ORDER_SHAPE};
    else
      orders = {order};
    std::unique_ptr<rs_plan> best;
    for (int o : orders) {
      std::unique_ptr<rs_plan> p(new rs_plan());
      rs::order_tensors(listed, o, &p->orig);
      for (int32_t i : p->orig) p->t.push_back(listed[size_t(i)]);
      p->world = world;
      p->g_coll = g_coll;
      p->A = A;
      rc = rs::solve_shard_size(p->t, p->world, p->g_coll, p->A, listing_only, &p->S);
      if (rc != RS_OK) return rc;
      if (!best || p->S < best->S) best = std::move(p);
    }
    std::unique_ptr<rs_plan>& p = best;
    std::vector<int64_t> starts;
    if (!rs::check_valid_shard(p->t, p->world, p->S, p->A, &starts)) return RS_EINVAL;
    finish_plan(p.get(), starts);
    *out = p.release();
    return RS_OK;
  } catch (const std::bad_alloc&) {
    return RS_ENOMEM;
  }
}

int rs_plan_create(const rs_tensor_desc* descs, int n, int world, int align_bytes, int min_itemsize,
                   int tensor_align_elems, rs_plan** out) {
  return rs_plan_create_ordered(descs, n, world, align_bytes, min_itemsize, tensor_align_elems,
                                RS_ORDER_DEFAULT, out);
}

int rs_plan_create_rooted(const rs_tensor_desc* descs, int n, int world, int align_bytes,
                          int min_itemsize, int tensor_align_elems, const int32_t* roots,
                          rs_plan** out) {
  if (!out) return RS_EINVAL;
  *out = nullptr;
  if (!roots) return RS_EINVAL;
  try {
    std::vector<rs::TensorHost> listed;
    int64_t g_coll = 0, A = 0;
    int rc = build_plan(descs, n, world, align_bytes, min_itemsize, tensor_align_elems, &listed,
                        &g_coll, &A);
    if (rc != RS_OK) return rc;
    std::unique_ptr<rs_plan> p(new rs_plan());
    p->world = world;
    p->g_coll = g_coll;
    p->A = A;
    std::vector<int64_t> starts;
    rc = rs::rooted_layout(listed, world, g_coll, A, roots, &p->orig, &starts, &p->S);
    if (rc != RS_OK) return rc;
    for (int32_t i : p->orig) p->t.push_back(listed[size_t(i)]);
    finish_plan(p.get(), starts);
    *out = p.release();
    return RS_OK;
  } catch (const std::bad_alloc&) {
    return RS_ENOMEM;
  }
}

int rs_select_roots(const rs_tensor_desc* descs, int n, int world, int32_t* roots, double* loads) {
  if (!descs || !roots || n <= 0 || world <= 0) return RS_EINVAL;
  try {
    std::vector<rs::TensorHost> t;
    const int rc = rs::describe_tensors(descs, n, &t);
    if (rc != RS_OK) return rc;
    rs::select_roots(t, world, roots, loads);
    return RS_OK;
  } catch (const std::bad_alloc&) {
    return RS_ENOMEM;
  }
}

int rs_shard_dim_granularity(const int64_t* shape, int ndim, int dim, int64_t g_user,
                             int64_t* g_out) {
  return rs::shard_dim_granularity(shape, ndim, dim, g_user, g_out);
}

void rs_plan_destroy(rs_plan* plan) {
  if (!plan) return;
  free_device_tables(&plan->dev);
  delete plan;
}

int rs_check_valid_shard(const rs_tensor_desc* descs, int n, int world, int align_bytes,
                         int min_itemsize, int tensor_align_elems, int64_t S) {
  try {
    std::vector<rs::TensorHost> t;
    int64_t g_coll = 0, A = 0;
    const int rc = build_plan(descs, n, world, align_bytes, min_itemsize, tensor_align_elems, &t,
                              &g_coll, &A);
    if (rc != RS_OK) return rc;
    if (S <= 0 || S % A != 0) return RS_EINVAL;
    if (S >= (int64_t(1) << 62) / world) return RS_EOVERFLOW;
    return rs::check_valid_shard(t, world, S, A, nullptr) ? 1 : 0;
  } catch (const std::bad_alloc&) {
    return RS_ENOMEM;
  }
}

int rs_plan_num_tensors(const rs_plan* plan) { return plan ? int(plan->t.size()) : RS_EINVAL; }
int rs_plan_world(const rs_plan* plan) { return plan ? int(plan->world) : RS_EINVAL; }
int64_t rs_plan_shard_elems(const rs_plan* plan) { return plan ? plan->S : RS_EINVAL; }
int64_t rs_plan_total_elems(const rs_plan* plan) { return plan ? plan->S * plan->world : RS_EINVAL; }
int64_t rs_plan_payload_elems(const rs_plan* plan) { return plan ? plan->payload : RS_EINVAL; }
int64_t rs_plan_padding_elems(const rs_plan* plan) {
  return plan ? plan->S * plan->world - plan->payload : RS_EINVAL;
}
int64_t rs_plan_num_scales(const rs_plan* plan) { return plan ? plan->num_scales : RS_EINVAL; }

int rs_plan_order(const rs_plan* plan, int32_t* out, int cap) {
  if (!plan || !out || cap < int(plan->t.size())) return RS_EINVAL;
  for (size_t j = 0; j < plan->t.size(); ++j) out[j] = plan->orig[j];
  return RS_OK;
}

int rs_plan_offsets(const rs_plan* plan, int64_t* out, int cap) {
  if (!plan || !out || cap < int(plan->t.size())) return RS_EINVAL;
  for (size_t j = 0; j < plan->t.size(); ++j) out[size_t(plan->orig[j])] = plan->t[j].ell;
  return RS_OK;
}

int rs_plan_scale_bases(const rs_plan* plan, int64_t* out, int cap) {
  if (!plan || !out || cap < int(plan->t.size()) + 1) return RS_EINVAL;
  for (size_t j = 0; j < plan->t.size(); ++j) out[size_t(plan->orig[j])] = plan->t[j].scale_base;
  out[plan->t.size()] = plan->num_scales;
  return RS_OK;
}

int rs_plan_scale_range(const rs_plan* plan, int rank, int64_t* lo, int64_t* hi) {
  if (!plan || !lo || !hi || rank < 0 || rank >= plan->world) return RS_EINVAL;
  *lo = plan->scale_begin[size_t(rank)];
  *hi = plan->scale_begin[size_t(rank) + 1];
  return RS_OK;
}

int64_t rs_plan_num_state_blocks(const rs_plan* plan) {
  if (!plan) return RS_EINVAL;
  return plan->all_state ? plan->num_state_blocks : RS_EUNSUPPORTED;
}

int rs_plan_state_bases(const rs_plan* plan, int64_t* out, int cap) {
  if (!plan || !out || cap < int(plan->t.size()) + 1) return RS_EINVAL;
  if (!plan->all_state) return RS_EUNSUPPORTED;
  for (size_t j = 0; j < plan->t.size(); ++j) out[size_t(plan->orig[j])] = plan->t[j].state_base;
  out[plan->t.size()] = plan->num_state_blocks;
  return RS_OK;
}

int rs_plan_state_range(const rs_plan* plan, int rank, int64_t* lo, int64_t* hi) {
  if (!plan || !lo || !hi || rank < 0 || rank >= plan->world) return RS_EINVAL;
  if (!plan->all_state) return RS_EUNSUPPORTED;
  *lo = plan->state_begin[size_t(rank)];
  *hi = plan->state_begin[size_t(rank) + 1];
  return RS_OK;
}

int rs_plan_rank_segments(const rs_plan* plan, int rank, rs_segment* out, int cap) {
  if (!plan || rank < 0 || rank >= plan->world || cap < 0 || (cap > 0 && !out)) return RS_EINVAL;
  const int64_t lo = int64_t(rank) * plan->S, hi = lo + plan->S;
  int count = 0;
  for (size_t i = 0; i < plan->t.size(); ++i) {
    const rs::TensorHost& h = plan->t[i];
    const int64_t a = h.ell > lo ? h.ell : lo;
    const int64_t b = h.ell + h.e < hi ? h.ell + h.e : hi;
    if (a >= b) continue;
    if (count < cap) {
      rs_segment s{};
      s.tensor = plan->orig[i];
      s.src_off = a - h.ell;
      s.dst_off = a - lo;
      s.n = b - a;
      out[count] = s;
    }
    ++count;
  }
  return count;
}

int rs_plan_upload(rs_plan* plan, int device) {
  if (!plan || device < 0) return RS_EINVAL;
  if (plan->S % 8 != 0) return RS_EUNSUPPORTED;  // bf16 rank regions must start 16-byte aligned
  // granule ids are 32-bit on the device and a granule is served by four workgroups
  if ((plan->S + rs::kGranule - 1) / rs::kGranule > (0x7fffffffLL / 4) / plan->world) return RS_EOVERFLOW;
  if (plan->dev.device >= 0) return plan->dev.device == device ? RS_OK : RS_EINVAL;
  int cur = -1;
  if (hipGetDevice(&cur) != hipSuccess) return RS_EHIP;
  if (cur != device && hipSetDevice(device) != hipSuccess) return RS_EHIP;
  int rc = rs::scratch_init(device);   // where this GPU keeps the fixed array of rs_pack_noalloc
  if (rc != RS_OK) {
    if (cur != device) (void)hipSetDevice(cur);
    return rc;
  }
  try {
    rs::build_host_tables(plan->t, plan->world, plan->S, plan->all_quant, plan->all_state,
                          &plan->host);
    rs::DeviceTables d;
    d.device = device;
    rc = upload(plan->host.tensors, &d.tensors);
    if (rc == RS_OK) rc = upload(plan->host.gran_first, &d.gran_first);
    if (rc == RS_OK) rc = upload(plan->host.items, &d.items);
    if (rc == RS_OK) rc = upload(plan->host.payload_gran, &d.payload_gran);
    if (rc == RS_OK) rc = upload(plan->host.padding_gran, &d.padding_gran);
    if (rc == RS_OK) rc = upload(plan->host.state_items, &d.state_items);
    if (rc == RS_OK) {
      plan->dev = d;
    } else {
      free_device_tables(&d);
    }
    // the big host mirrors are not needed again
    std::vector<int32_t>().swap(plan->host.gran_first);
    std::vector<rs::QItem>().swap(plan->host.items);
    std::vector<rs::GranRef>().swap(plan->host.payload_gran);
    std::vector<int32_t>().swap(plan->host.padding_gran);
    std::vector<rs::Item>().swap(plan->host.state_items);
  } catch (const std::bad_alloc&) {
    rc = RS_ENOMEM;
  }
  if (cur != device) (void)hipSetDevice(cur);
  return rc;
}

int rs_tensor_table_create(const rs_plan* plan, const void* const* ptrs, rs_tensor_table** out) {
  if (!out) return RS_EINVAL;
  *out = nullptr;
  if (!ptrs) return RS_EINVAL;
  const int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  const int n = int(plan->t.size());
  for (int i = 0; i < n; ++i) {
    if (!ptrs[i]) return RS_EINVAL;
    if (reinterpret_cast<uintptr_t>(ptrs[i]) & 1) return RS_EALIGN;  // bf16 element alignment
  }
  rs_tensor_table* tab = new (std::nothrow) rs_tensor_table();
  if (!tab) return RS_ENOMEM;
  tab->device = plan->dev.device;
  tab->owner = plan;
  tab->n = n;
  for (int i = 0; i < n; ++i) tab->low_bits |= unsigned(reinterpret_cast<uintptr_t>(ptrs[i]) & 15);
  if (hipMalloc(reinterpret_cast<void**>(&tab->ptrs), sizeof(void*) * n) != hipSuccess) {
    delete tab;
    return RS_ENOMEM;
  }
  // device table in buffer order, like the tensor records
  int copied = RS_ENOMEM;
  try {
    std::vector<const void*> ordered(size_t(n), nullptr);
    for (int j = 0; j < n; ++j) ordered[size_t(j)] = ptrs[plan->orig[size_t(j)]];
    copied = hipMemcpy(tab->ptrs, ordered.data(), sizeof(void*) * n, hipMemcpyHostToDevice) == hipSuccess
                 ? RS_OK
                 : RS_EHIP;
  } catch (const std::bad_alloc&) {
  }
  if (copied != RS_OK) {
    (void)hipFree(tab->ptrs);
    delete tab;
    return copied;
  }
  *out = tab;
  return RS_OK;
}

void rs_tensor_table_destroy(rs_tensor_table* table) {
  if (!table) return;
  if (table->ptrs) (void)hipFree(table->ptrs);
  delete table;
}

// shared body of the group-level operators on the bf16 DBuffer
static int group_op(int op, const rs_plan* plan, const rs_tensor_table* tab, const void* dbuf,
                    float alpha, void* stream, int64_t region_stride = 0) {
  int rc = check_device(plan);
  if (rc == RS_OK && op != rs::kGroupScale) rc = check_table(plan, tab);
  if (rc != RS_OK) return rc;
  if (!dbuf) return RS_EINVAL;
  if (!aligned16(dbuf)) return RS_EALIGN;
  if (alpha != alpha || alpha - alpha != 0.0f) return RS_EINVAL;  // NaN or infinite factor
  if (region_stride == 0) region_stride = plan->S;
  if (region_stride < plan->S) return RS_EINVAL;
  if (region_stride % 8 != 0) return RS_EALIGN;
  return rs::launch_group_op(op, plan->dev, int(plan->t.size()), tab ? tab->ptrs : nullptr,
                             const_cast<void*>(dbuf), alpha, plan->S, plan->host.granules_per_rank,
                             region_stride, plan->host.n_payload_gran, plan->host.n_padding_gran,
                             static_cast<hipStream_t>(stream));
}

int rs_pack(const rs_plan* plan, const rs_tensor_table* src, void* dbuf, void* stream) {
  return group_op(rs::kGroupPack, plan, src, dbuf, 1.0f, stream);
}

int rs_pack_noalloc(const rs_plan* plan, const void* const* src_ptrs, void* dbuf, void* stream) {
  const int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!src_ptrs || !dbuf) return RS_EINVAL;
  if (!aligned16(dbuf)) return RS_EALIGN;
  const int n = int(plan->t.size());
  if (n > RS_NOALLOC_MAX_TENSORS) return RS_ETOOBIG;
  for (int i = 0; i < n; ++i) {
    if (!src_ptrs[i]) return RS_EINVAL;
    if (reinterpret_cast<uintptr_t>(src_ptrs[i]) & 1) return RS_EALIGN;  // bf16 element alignment
  }
  return rs::launch_pack_staged(plan->dev, n, src_ptrs, plan->orig.data(), dbuf, plan->S,
                                plan->host.granules_per_rank, plan->host.n_payload_gran,
                                plan->host.n_padding_gran, static_cast<hipStream_t>(stream));
}

int rs_unpack_bf16(const rs_plan* plan, const void* dbuf, const rs_tensor_table* dst, void* stream) {
  return group_op(rs::kGroupUnpack, plan, dst, dbuf, 1.0f, stream);
}

int rs_pack_strided(const rs_plan* plan, const rs_tensor_table* src, void* dbuf, int64_t region_stride,
                    void* stream) {
  if (region_stride <= 0) return RS_EINVAL;
  return group_op(rs::kGroupPack, plan, src, dbuf, 1.0f, stream, region_stride);
}

int rs_unpack_bf16_strided(const rs_plan* plan, const void* dbuf, int64_t region_stride,
                           const rs_tensor_table* dst, void* stream) {
  if (region_stride <= 0) return RS_EINVAL;
  return group_op(rs::kGroupUnpack, plan, dst, dbuf, 1.0f, stream, region_stride);
}

int rs_pack_scaled(const rs_plan* plan, const rs_tensor_table* src, float alpha, void* dbuf,
                   void* stream) {
  return group_op(rs::kGroupPackScaled, plan, src, dbuf, alpha, stream);
}

int rs_group_add(const rs_plan* plan, const rs_tensor_table* src, float alpha, void* dbuf,
                 void* stream) {
  return group_op(rs::kGroupAdd, plan, src, dbuf, alpha, stream);
}

int rs_group_scale(const rs_plan* plan, float alpha, void* dbuf, void* stream) {
  return group_op(rs::kGroupScale, plan, nullptr, dbuf, alpha, stream);
}

int rs_group_zero(const rs_plan* plan, void* dbuf, void* stream) {
  const int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!dbuf) return RS_EINVAL;
  if (!aligned16(dbuf)) return RS_EALIGN;
  return rs::launch_fill_zero(dbuf, plan->S * plan->world * 2, static_cast<hipStream_t>(stream));
}

int rs_reduce_rows(const rs_plan* plan, int rank, const void* partials, int rows, int64_t row_stride,
                   float* out, void* stream) {
  const int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!partials || !out || rank < 0 || rank >= plan->world || rows < 1 || rows > (1 << 24) ||
      row_stride < plan->S)
    return RS_EINVAL;
  if (!aligned16(partials) || !aligned16(out) || row_stride % 8 != 0) return RS_EALIGN;
  return rs::launch_shard_reduce(plan->dev, int(plan->t.size()), partials, row_stride, out, plan->S,
                                 plan->host.granules_per_rank, rank, rows, nullptr, 0,
                                 static_cast<hipStream_t>(stream));
}

int rs_partials_batch_create(const rs_plan* plan, int rank, int count, const void* const* partials,
                             int64_t row_stride, float* const* outs, rs_partials_batch** out) {
  if (!out) return RS_EINVAL;
  *out = nullptr;
  const int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!partials || !outs || count <= 0 || count > 65535 || rank < 0 || rank >= plan->world ||
      row_stride < plan->S)
    return RS_EINVAL;
  if (row_stride % 8 != 0) return RS_EALIGN;
  Staging host(size_t(count) * 2);
  if (!host.data) return RS_ENOMEM;
  for (int u = 0; u < count; ++u) {
    if (!partials[u] || !outs[u]) return RS_EINVAL;
    if (!aligned16(partials[u]) || !aligned16(outs[u])) return RS_EALIGN;
    host[size_t(u)] = const_cast<void*>(partials[u]);
    host[size_t(count) + u] = outs[u];
  }
  rs_partials_batch* b = new (std::nothrow) rs_partials_batch();
  if (!b) return RS_ENOMEM;
  b->owner = plan;
  b->rank = rank;
  b->count = count;
  b->row_stride = row_stride;
  const size_t bytes = host.size() * sizeof(void*);
  if (hipMalloc(reinterpret_cast<void**>(&b->ptrs), bytes) != hipSuccess) {
    delete b;
    return RS_ENOMEM;
  }
  if (hipMemcpy(b->ptrs, host.data.get(), bytes, hipMemcpyHostToDevice) != hipSuccess) {
    (void)hipFree(b->ptrs);
    delete b;
    return RS_EHIP;
  }
  *out = b;
  return RS_OK;
}

void rs_partials_batch_destroy(rs_partials_batch* batch) {
  if (!batch) return;
  if (batch->ptrs) (void)hipFree(batch->ptrs);
  delete batch;
}

int rs_reduce_batch(const rs_plan* plan, const rs_partials_batch* batch, void* stream) {
  const int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!batch || batch->owner != plan || !batch->ptrs) return RS_EINVAL;
  return rs::launch_shard_reduce(plan->dev, int(plan->t.size()), nullptr, batch->row_stride, nullptr,
                                 plan->S, plan->host.granules_per_rank, batch->rank, int(plan->world),
                                 batch->ptrs, batch->count, static_cast<hipStream_t>(stream));
}

int rs_reduce(const rs_plan* plan, int rank, const void* partials, int64_t row_stride, float* out,
              void* stream) {
  return rs_reduce_rows(plan, rank, partials, plan ? int(plan->world) : 0, row_stride, out, stream);
}

int rs_quantize(const rs_plan* plan, int rank, const void* shard, uint8_t* codes, float* scales,
                void* stream) {
  const int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!plan->all_quant) return RS_EUNSUPPORTED;
  if (!shard || !codes || !scales || rank < -1 || rank >= plan->world) return RS_EINVAL;
  if (!aligned16(shard) || !aligned16(codes) || (reinterpret_cast<uintptr_t>(scales) & 3))
    return RS_EALIGN;
  const std::vector<int64_t>& ib = plan->host.item_begin;
  int64_t first = 0, count = ib[size_t(plan->world)], elem_base = 0, scale_off = 0;
  if (rank >= 0) {
    first = ib[size_t(rank)];
    count = ib[size_t(rank) + 1] - first;
    elem_base = int64_t(rank) * plan->S;
    scale_off = plan->scale_begin[size_t(rank)];
  }
  return rs::launch_block_quant(plan->dev, first, count, shard, codes, scales, nullptr, 0, elem_base,
                                scale_off, static_cast<hipStream_t>(stream));
}

int rs_reduce_quantize(const rs_plan* plan, int rank, const void* partials, int64_t row_stride,
                       uint8_t* codes, float* scales, float* mean_out, void* stream) {
  const int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!plan->all_quant) return RS_EUNSUPPORTED;
  if (!partials || !codes || !scales || rank < 0 || rank >= plan->world || row_stride < plan->S)
    return RS_EINVAL;
  if (!aligned16(partials) || !aligned16(codes) || !aligned16(mean_out) || row_stride % 8 != 0 ||
      (reinterpret_cast<uintptr_t>(scales) & 3))
    return RS_EALIGN;
  const std::vector<int64_t>& ib = plan->host.item_begin;
  return rs::launch_reduce_quant(plan->dev, ib[size_t(rank)], ib[size_t(rank) + 1] - ib[size_t(rank)],
                                 partials, row_stride, codes, scales, mean_out, nullptr, nullptr, 0,
                                 false, int64_t(rank) * plan->S, plan->scale_begin[size_t(rank)],
                                 int(plan->world), static_cast<hipStream_t>(stream));
}

int rs_reduce_quantize_batch(const rs_plan* plan, const rs_partials_batch* in,
                             const rs_shard_batch* out, int write_means, void* stream) {
  const int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!plan->all_quant) return RS_EUNSUPPORTED;
  if (!in || !out || in->owner != plan || out->owner != plan || !in->ptrs || !out->ptrs ||
      in->rank != out->rank || in->count != out->count)
    return RS_EINVAL;
  const int rank = in->rank;
  const std::vector<int64_t>& ib = plan->host.item_begin;
  return rs::launch_reduce_quant(plan->dev, ib[size_t(rank)], ib[size_t(rank) + 1] - ib[size_t(rank)],
                                 nullptr, in->row_stride, nullptr, nullptr, nullptr, in->ptrs,
                                 out->ptrs, in->count, write_means != 0, int64_t(rank) * plan->S,
                                 plan->scale_begin[size_t(rank)], int(plan->world),
                                 static_cast<hipStream_t>(stream));
}

// checks the hyper-parameters and derives the step's fp32 constants: each is evaluated in
// double precision and rounded once
static int adam8_consts(const rs_adam8_hyper* hyper, rs::Adam8Consts* c) {
  if (!hyper) return RS_EINVAL;
  const rs_adam8_hyper& h = *hyper;
  if (!std::isfinite(h.lr) || !std::isfinite(h.weight_decay) || !(h.beta1 >= 0.0 && h.beta1 < 1.0) ||
      !(h.beta2 >= 0.0 && h.beta2 < 1.0) || !(h.eps > 0.0) || !std::isfinite(h.eps) || h.step < 1)
    return RS_EINVAL;
  const double bc1 = 1.0 - std::pow(h.beta1, double(h.step));
  const double bc2 = 1.0 - std::pow(h.beta2, double(h.step));
  c->beta1 = float(h.beta1);
  c->beta2 = float(h.beta2);
  c->one_minus_beta1 = float(1.0 - h.beta1);
  c->one_minus_beta2 = float(1.0 - h.beta2);
  c->eps = float(h.eps);
  c->step_size = float(h.lr / bc1);
  c->bc2_sqrt = float(std::sqrt(bc2));
  c->decay = float(1.0 - h.lr * h.weight_decay);
  if (!std::isfinite(c->step_size) || !(c->bc2_sqrt > 0.0f)) return RS_EINVAL;
  c->bc2_sqrt_rcp = 1.0 / double(c->bc2_sqrt);
  return RS_OK;
}

static int adam8_check_buffers(const rs_plan* plan, int rank, const float* grad, const float* master,
                               const void* param_bf16, const int8_t* m_codes, const uint8_t* v_codes,
                               const float* m_absmax, const float* v_absmax) {
  if (!grad || !master || !m_codes || !v_codes) return RS_EINVAL;
  const int64_t nblk = plan->state_begin[size_t(rank) + 1] - plan->state_begin[size_t(rank)];
  if (nblk > 0 && (!m_absmax || !v_absmax)) return RS_EINVAL;
  if (!aligned16(grad) || !aligned16(master) || !aligned16(param_bf16) || !aligned16(m_codes) ||
      !aligned16(v_codes) || (reinterpret_cast<uintptr_t>(m_absmax) & 3) ||
      (reinterpret_cast<uintptr_t>(v_absmax) & 3))
    return RS_EALIGN;
  return RS_OK;
}

int rs_adam8_step(const rs_plan* plan, int rank, const rs_adam8_hyper* hyper, const float* grad,
                  float* master, void* param_bf16, int8_t* m_codes, uint8_t* v_codes,
                  float* m_absmax, float* v_absmax, void* stream) {
  int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!plan->all_state) return RS_EUNSUPPORTED;
  if (rank < 0 || rank >= plan->world) return RS_EINVAL;
  rs::Adam8Consts c;
  rc = adam8_consts(hyper, &c);
  if (rc == RS_OK)
    rc = adam8_check_buffers(plan, rank, grad, master, param_bf16, m_codes, v_codes, m_absmax, v_absmax);
  if (rc != RS_OK) return rc;
  const std::vector<int64_t>& ib = plan->host.state_item_begin;
  return rs::launch_adam8_step(plan->dev, ib[size_t(rank)], ib[size_t(rank) + 1] - ib[size_t(rank)],
                               grad, master, param_bf16, m_codes, v_codes, m_absmax, v_absmax, nullptr,
                               0, int64_t(rank) * plan->S, plan->state_begin[size_t(rank)], c,
                               static_cast<hipStream_t>(stream));
}

static int state_codec(bool quantise, const rs_plan* plan, int rank, float* x, void* codes,
                       float* absmax, int is_unsigned, void* stream) {
  const int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!plan->all_state) return RS_EUNSUPPORTED;
  if (!x || !codes || rank < 0 || rank >= plan->world || (is_unsigned != 0 && is_unsigned != 1))
    return RS_EINVAL;
  const int64_t nblk = plan->state_begin[size_t(rank) + 1] - plan->state_begin[size_t(rank)];
  if (nblk > 0 && !absmax) return RS_EINVAL;
  if (!aligned16(x) || !aligned16(codes) || (reinterpret_cast<uintptr_t>(absmax) & 3)) return RS_EALIGN;
  const std::vector<int64_t>& ib = plan->host.state_item_begin;
  return rs::launch_state_codec(quantise, plan->dev, ib[size_t(rank)],
                                ib[size_t(rank) + 1] - ib[size_t(rank)], x,
                                static_cast<uint8_t*>(codes), absmax, is_unsigned != 0,
                                int64_t(rank) * plan->S, plan->state_begin[size_t(rank)],
                                static_cast<hipStream_t>(stream));
}

int rs_state_quantize(const rs_plan* plan, int rank, const float* src, int is_unsigned, void* codes,
                      float* absmax, void* stream) {
  return state_codec(true, plan, rank, const_cast<float*>(src), codes, absmax, is_unsigned, stream);
}

int rs_state_dequantize(const rs_plan* plan, int rank, const void* codes, const float* absmax,
                        int is_unsigned, float* dst, void* stream) {
  return state_codec(false, plan, rank, dst, const_cast<void*>(codes), const_cast<float*>(absmax),
                     is_unsigned, stream);
}

int rs_adam8_batch_create(const rs_plan* plan, int rank, int count, const float* const* grads,
                          float* const* masters, void* const* params_bf16, int8_t* const* m_codes,
                          uint8_t* const* v_codes, float* const* m_absmax, float* const* v_absmax,
                          rs_adam8_batch** out) {
  if (!out) return RS_EINVAL;
  *out = nullptr;
  const int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!plan->all_state) return RS_EUNSUPPORTED;
  if (!grads || !masters || !m_codes || !v_codes || !m_absmax || !v_absmax || count <= 0 ||
      count > 65535 || rank < 0 || rank >= plan->world)
    return RS_EINVAL;
  Staging host(size_t(count) * 7);
  if (!host.data) return RS_ENOMEM;
  for (int u = 0; u < count; ++u) {
    void* const param = params_bf16 ? params_bf16[u] : nullptr;
    const int brc = adam8_check_buffers(plan, rank, grads[u], masters[u], param, m_codes[u], v_codes[u],
                                        m_absmax[u], v_absmax[u]);
    if (brc != RS_OK) return brc;
    host[size_t(u)] = const_cast<float*>(grads[u]);
    host[size_t(count) + u] = masters[u];
    host[size_t(count) * 2 + u] = param;
    host[size_t(count) * 3 + u] = m_codes[u];
    host[size_t(count) * 4 + u] = v_codes[u];
    host[size_t(count) * 5 + u] = m_absmax[u];
    host[size_t(count) * 6 + u] = v_absmax[u];
  }
  rs_adam8_batch* b = new (std::nothrow) rs_adam8_batch();
  if (!b) return RS_ENOMEM;
  b->owner = plan;
  b->rank = rank;
  b->count = count;
  const size_t bytes = host.size() * sizeof(void*);
  if (hipMalloc(reinterpret_cast<void**>(&b->ptrs), bytes) != hipSuccess) {
    delete b;
    return RS_ENOMEM;
  }
  if (hipMemcpy(b->ptrs, host.data.get(), bytes, hipMemcpyHostToDevice) != hipSuccess) {
    (void)hipFree(b->ptrs);
    delete b;
    return RS_EHIP;
  }
  *out = b;
  return RS_OK;
}

void rs_adam8_batch_destroy(rs_adam8_batch* batch) {
  if (!batch) return;
  if (batch->ptrs) (void)hipFree(batch->ptrs);
  delete batch;
}

int rs_adam8_step_batch(const rs_plan* plan, const rs_adam8_batch* batch, const rs_adam8_hyper* hyper,
                        void* stream) {
  int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!batch || batch->owner != plan || !batch->ptrs) return RS_EINVAL;
  rs::Adam8Consts c;
  rc = adam8_consts(hyper, &c);
  if (rc != RS_OK) return rc;
  const int rank = batch->rank;
  const std::vector<int64_t>& ib = plan->host.state_item_begin;
  return rs::launch_adam8_step(plan->dev, ib[size_t(rank)], ib[size_t(rank) + 1] - ib[size_t(rank)],
                               nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                               batch->ptrs, batch->count, int64_t(rank) * plan->S,
                               plan->state_begin[size_t(rank)], c, static_cast<hipStream_t>(stream));
}

int rs_shard_batch_create(const rs_plan* plan, int rank, int count, const void* const* shards,
                          uint8_t* const* codes, float* const* scales, rs_shard_batch** out) {
  if (!out) return RS_EINVAL;
  *out = nullptr;
  const int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!plan->all_quant) return RS_EUNSUPPORTED;
  if (!shards || !codes || !scales || count <= 0 || count > 65535 || rank < 0 || rank >= plan->world)
    return RS_EINVAL;
  const bool has_scales = plan->scale_begin[size_t(rank) + 1] > plan->scale_begin[size_t(rank)];
  Staging host(size_t(count) * 3);
  if (!host.data) return RS_ENOMEM;
  for (int u = 0; u < count; ++u) {
    if (!shards[u] || !codes[u] || (!scales[u] && has_scales)) return RS_EINVAL;
    if (!aligned16(shards[u]) || !aligned16(codes[u]) || (reinterpret_cast<uintptr_t>(scales[u]) & 3))
      return RS_EALIGN;
    host[size_t(u)] = const_cast<void*>(shards[u]);
    host[size_t(count) + u] = codes[u];
    host[size_t(count) * 2 + u] = scales[u];
  }
  rs_shard_batch* b = new (std::nothrow) rs_shard_batch();
  if (!b) return RS_ENOMEM;
  b->owner = plan;
  b->rank = rank;
  b->count = count;
  const size_t bytes = host.size() * sizeof(void*);
  if (hipMalloc(reinterpret_cast<void**>(&b->ptrs), bytes) != hipSuccess) {
    delete b;
    return RS_ENOMEM;
  }
  if (hipMemcpy(b->ptrs, host.data.get(), bytes, hipMemcpyHostToDevice) != hipSuccess) {
    (void)hipFree(b->ptrs);
    delete b;
    return RS_EHIP;
  }
  *out = b;
  return RS_OK;
}

void rs_shard_batch_destroy(rs_shard_batch* batch) {
  if (!batch) return;
  if (batch->ptrs) (void)hipFree(batch->ptrs);
  delete batch;
}

int rs_quantize_batch(const rs_plan* plan, const rs_shard_batch* batch, void* stream) {
  const int rc = check_device(plan);
  if (rc != RS_OK) return rc;
  if (!batch || batch->owner != plan || !batch->ptrs) return RS_EINVAL;
  const std::vector<int64_t>& ib = plan->host.item_begin;
  const int64_t first = ib[size_t(batch->rank)];
  return rs::launch_block_quant(plan->dev, first, ib[size_t(batch->rank) + 1] - first, nullptr,
                                nullptr, nullptr, batch->ptrs, batch->count,
                                int64_t(batch->rank) * plan->S, plan->scale_begin[size_t(batch->rank)],
                                static_cast<hipStream_t>(stream));
}

// shared body of the four dequant_unpack entry points
static int dequant_unpack(bool f32_out, const rs_plan* plan, const uint8_t* codes, int64_t region_stride,
                          const float* scales, const rs_tensor_table* dst, void* stream) {
  int rc = check_device(plan);
  if (rc == RS_OK) rc = check_table(plan, dst);
  if (rc != RS_OK) return rc;
  if (!plan->all_quant) return RS_EUNSUPPORTED;
  if (!codes || !scales || region_stride < plan->S) return RS_EINVAL;
  if (!aligned16(codes) || (reinterpret_cast<uintptr_t>(scales) & 3) || region_stride % 8 != 0 ||
      (f32_out && (dst->low_bits & 3)))
    return RS_EALIGN;
  return rs::launch_dequant_unpack(f32_out, plan->dev, int(plan->t.size()), plan->host.n_payload_gran,
                                   codes, scales, dst->ptrs, plan->S, plan->host.granules_per_rank,
                                   region_stride, static_cast<hipStream_t>(stream));
}

int rs_unpack(const rs_plan* plan, const uint8_t* codes, const float* scales,
              const rs_tensor_table* dst, void* stream) {
  return dequant_unpack(false, plan, codes, plan ? plan->S : 0, scales, dst, stream);
}

int rs_unpack_f32(const rs_plan* plan, const uint8_t* codes, const float* scales,
                  const rs_tensor_table* dst, void* stream) {
  return dequant_unpack(true, plan, codes, plan ? plan->S : 0, scales, dst, stream);
}

int rs_unpack_strided(const rs_plan* plan, const uint8_t* codes, int64_t region_stride,
                      const float* scales, const rs_tensor_table* dst, void* stream) {
  if (region_stride <= 0) return RS_EINVAL;
  return dequant_unpack(false, plan, codes, region_stride, scales, dst, stream);
}

int rs_unpack_f32_strided(const rs_plan* plan, const uint8_t* codes, int64_t region_stride,
                          const float* scales, const rs_tensor_table* dst, void* stream) {
  if (region_stride <= 0) return RS_EINVAL;
  return dequant_unpack(true, plan, codes, region_stride, scales, dst, stream);
}

int rs_copy_probe(void* dst, const void* src, int64_t bytes, void* stream) {
  if (!dst || !src || bytes < 0 || bytes % 16 != 0) return RS_EINVAL;
  if (!aligned16(dst) || !aligned16(src)) return RS_EALIGN;
  return rs::launch_copy_probe(dst, src, bytes, static_cast<hipStream_t>(stream));
}

}  // extern "C"
