"""ctypes binding of libraggedshard.so: the same entry points as include/raggedshard.h, with
Python argument marshalling and nothing else.  torch tensors are used for device memory and
streams only; every step of the path runs in the library's kernels.  There is no fallback:
a missing library or a failing call raises."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Sequence, Tuple

LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libraggedshard.so")

RS_BLOCK_1x128, RS_BLOCK_128x128, RS_BLOCK_WHOLE, RS_BLOCK_EXPLICIT, RS_BLOCK_32x32 = 0, 1, 2, 3, 4
RS_ORDER_DEFAULT, RS_ORDER_BLOCK_SIZE, RS_ORDER_SHAPE, RS_ORDER_BEST = 0, 1, 2, 3
RS_UNITS_LISTING = 256
RS_OK, RS_EINVAL, RS_EOVERFLOW, RS_ENOMEM, RS_EALIGN, RS_EUNSUPPORTED, RS_EHIP, RS_ENOTUPLOADED, RS_ETOOBIG = (
    0, -1, -2, -3, -4, -5, -6, -7, -8)
RS_NOALLOC_MAX_TENSORS = 4096

EXPORTS = [
    "rs_version", "rs_strerror", "rs_plan_create", "rs_plan_destroy", "rs_check_valid_shard",
    "rs_plan_num_tensors", "rs_plan_world", "rs_plan_shard_elems", "rs_plan_total_elems",
    "rs_plan_payload_elems", "rs_plan_padding_elems", "rs_plan_num_scales", "rs_plan_offsets",
    "rs_plan_scale_bases", "rs_plan_scale_range", "rs_plan_rank_segments", "rs_plan_upload",
    "rs_tensor_table_create", "rs_tensor_table_destroy", "rs_pack", "rs_unpack_bf16", "rs_reduce",
    "rs_quantize", "rs_unpack", "rs_copy_probe", "rs_shard_batch_create", "rs_shard_batch_destroy",
    "rs_quantize_batch", "rs_plan_create_ordered", "rs_plan_order",
    "rs_pack_scaled", "rs_group_add", "rs_group_scale", "rs_group_zero",
    "rs_plan_num_state_blocks", "rs_plan_state_bases", "rs_plan_state_range", "rs_adam8_step",
    "rs_adam8_batch_create", "rs_adam8_batch_destroy", "rs_adam8_step_batch", "rs_unpack_f32",
    "rs_state_quantize", "rs_state_dequantize", "rs_pack_strided", "rs_unpack_bf16_strided",
    "rs_plan_create_rooted", "rs_select_roots", "rs_shard_dim_granularity", "rs_reduce_quantize", "rs_reduce_quantize_batch",
    "rs_reduce_rows", "rs_pack_noalloc", "rs_partials_batch_create", "rs_partials_batch_destroy",
    "rs_reduce_batch", "rs_unpack_strided", "rs_unpack_f32_strided",
]


class rs_tensor_desc(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64), ("block_mode", C.c_int32),
                ("reserved", C.c_int32), ("g_explicit", C.c_int64)]


class rs_segment(C.Structure):
    _fields_ = [("tensor", C.c_int32), ("reserved", C.c_int32), ("src_off", C.c_int64),
                ("dst_off", C.c_int64), ("n", C.c_int64)]


class rs_adam8_hyper(C.Structure):
    _fields_ = [("lr", C.c_double), ("beta1", C.c_double), ("beta2", C.c_double), ("eps", C.c_double),
                ("weight_decay", C.c_double), ("step", C.c_int64)]


class RaggedShardError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {rs_strerror(code)} ({code})")


if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2602_22437_amd.build`; "
                      "there is no fallback path")
_lib = C.CDLL(LIB_PATH)

_P = C.c_void_p
_lib.rs_version.restype = C.c_int
_lib.rs_strerror.restype = C.c_char_p
_lib.rs_strerror.argtypes = [C.c_int]
_lib.rs_plan_create.argtypes = [C.POINTER(rs_tensor_desc), C.c_int, C.c_int, C.c_int, C.c_int, C.c_int,
                                C.POINTER(_P)]
_lib.rs_plan_create_ordered.argtypes = [C.POINTER(rs_tensor_desc), C.c_int, C.c_int, C.c_int, C.c_int,
                                        C.c_int, C.c_int, C.POINTER(_P)]
_lib.rs_plan_create_rooted.argtypes = [C.POINTER(rs_tensor_desc), C.c_int, C.c_int, C.c_int, C.c_int,
                                       C.c_int, C.POINTER(C.c_int32), C.POINTER(_P)]
_lib.rs_select_roots.argtypes = [C.POINTER(rs_tensor_desc), C.c_int, C.c_int, C.POINTER(C.c_int32),
                                 C.POINTER(C.c_double)]
_lib.rs_shard_dim_granularity.argtypes = [C.POINTER(C.c_int64), C.c_int, C.c_int, C.c_int64,
                                          C.POINTER(C.c_int64)]
_lib.rs_plan_order.argtypes = [_P, C.POINTER(C.c_int32), C.c_int]
_lib.rs_plan_destroy.argtypes = [_P]
_lib.rs_plan_destroy.restype = None
_lib.rs_check_valid_shard.argtypes = [C.POINTER(rs_tensor_desc), C.c_int, C.c_int, C.c_int, C.c_int,
                                      C.c_int, C.c_int64]
for _name in ("rs_plan_num_tensors", "rs_plan_world"):
    getattr(_lib, _name).argtypes = [_P]
    getattr(_lib, _name).restype = C.c_int
for _name in ("rs_plan_shard_elems", "rs_plan_total_elems", "rs_plan_payload_elems",
              "rs_plan_padding_elems", "rs_plan_num_scales"):
    getattr(_lib, _name).argtypes = [_P]
    getattr(_lib, _name).restype = C.c_int64
_lib.rs_plan_offsets.argtypes = [_P, C.POINTER(C.c_int64), C.c_int]
_lib.rs_plan_scale_bases.argtypes = [_P, C.POINTER(C.c_int64), C.c_int]
_lib.rs_plan_scale_range.argtypes = [_P, C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
_lib.rs_plan_rank_segments.argtypes = [_P, C.c_int, C.POINTER(rs_segment), C.c_int]
_lib.rs_plan_upload.argtypes = [_P, C.c_int]
_lib.rs_tensor_table_create.argtypes = [_P, C.POINTER(_P), C.POINTER(_P)]
_lib.rs_tensor_table_destroy.argtypes = [_P]
_lib.rs_tensor_table_destroy.restype = None
_lib.rs_pack.argtypes = [_P, _P, _P, _P]
_lib.rs_unpack_bf16.argtypes = [_P, _P, _P, _P]
_lib.rs_pack_noalloc.argtypes = [_P, C.POINTER(_P), _P, _P]
_lib.rs_pack_strided.argtypes = [_P, _P, _P, C.c_int64, _P]
_lib.rs_unpack_bf16_strided.argtypes = [_P, _P, C.c_int64, _P, _P]
_lib.rs_pack_scaled.argtypes = [_P, _P, C.c_float, _P, _P]
_lib.rs_group_add.argtypes = [_P, _P, C.c_float, _P, _P]
_lib.rs_group_scale.argtypes = [_P, C.c_float, _P, _P]
_lib.rs_group_zero.argtypes = [_P, _P, _P]
_lib.rs_reduce.argtypes = [_P, C.c_int, _P, C.c_int64, _P, _P]
_lib.rs_reduce_rows.argtypes = [_P, C.c_int, _P, C.c_int, C.c_int64, _P, _P]
_lib.rs_partials_batch_create.argtypes = [_P, C.c_int, C.c_int, C.POINTER(_P), C.c_int64, C.POINTER(_P),
                                          C.POINTER(_P)]
_lib.rs_partials_batch_destroy.argtypes = [_P]
_lib.rs_partials_batch_destroy.restype = None
_lib.rs_reduce_batch.argtypes = [_P, _P, _P]
_lib.rs_quantize.argtypes = [_P, C.c_int, _P, _P, _P, _P]
_lib.rs_reduce_quantize.argtypes = [_P, C.c_int, _P, C.c_int64, _P, _P, _P, _P]
_lib.rs_reduce_quantize_batch.argtypes = [_P, _P, _P, C.c_int, _P]
_lib.rs_unpack.argtypes = [_P, _P, _P, _P, _P]
_lib.rs_unpack_f32.argtypes = [_P, _P, _P, _P, _P]
_lib.rs_unpack_strided.argtypes = [_P, _P, C.c_int64, _P, _P, _P]
_lib.rs_unpack_f32_strided.argtypes = [_P, _P, C.c_int64, _P, _P, _P]
_lib.rs_shard_batch_create.argtypes = [_P, C.c_int, C.c_int, C.POINTER(_P), C.POINTER(_P), C.POINTER(_P),
                                       C.POINTER(_P)]
_lib.rs_shard_batch_destroy.argtypes = [_P]
_lib.rs_shard_batch_destroy.restype = None
_lib.rs_quantize_batch.argtypes = [_P, _P, _P]
_lib.rs_copy_probe.argtypes = [_P, _P, C.c_int64, _P]
_lib.rs_plan_num_state_blocks.argtypes = [_P]
_lib.rs_plan_num_state_blocks.restype = C.c_int64
_lib.rs_plan_state_bases.argtypes = [_P, C.POINTER(C.c_int64), C.c_int]
_lib.rs_plan_state_range.argtypes = [_P, C.c_int, C.POINTER(C.c_int64), C.POINTER(C.c_int64)]
_lib.rs_adam8_step.argtypes = [_P, C.c_int, C.POINTER(rs_adam8_hyper), _P, _P, _P, _P, _P, _P, _P, _P]
_lib.rs_state_quantize.argtypes = [_P, C.c_int, _P, C.c_int, _P, _P, _P]
_lib.rs_state_dequantize.argtypes = [_P, C.c_int, _P, _P, C.c_int, _P, _P]
_lib.rs_adam8_batch_create.argtypes = [_P, C.c_int, C.c_int] + [C.POINTER(_P)] * 7 + [C.POINTER(_P)]
_lib.rs_adam8_batch_destroy.argtypes = [_P]
_lib.rs_adam8_batch_destroy.restype = None
_lib.rs_adam8_step_batch.argtypes = [_P, _P, C.POINTER(rs_adam8_hyper), _P]


def _check(code: int, where: str) -> int:
    if code < 0:
        raise RaggedShardError(code, where)
    return code


def _descs(tensors: Sequence[Tuple]) -> "C.Array":
    arr = (rs_tensor_desc * max(1, len(tensors)))()
    for i, t in enumerate(tensors):
        rows, cols, mode = t[0], t[1], t[2]
        arr[i] = rs_tensor_desc(int(rows), int(cols), int(mode), 0, int(t[3]) if len(t) > 3 else 0)
    return arr


def _ptr(x) -> int:
    """Device (or host) address of a torch tensor, or a raw integer address."""
    return int(x.data_ptr()) if hasattr(x, "data_ptr") else int(x)


def _stream(stream) -> int:
    if stream is None:
        import torch
        return int(torch.cuda.current_stream().cuda_stream)
    return int(getattr(stream, "cuda_stream", stream))


# ---- same names as the C ABI ---------------------------------------------------------------

def rs_version() -> int:
    return _lib.rs_version()


def rs_strerror(code: int) -> str:
    return _lib.rs_strerror(int(code)).decode()


def rs_plan_create(tensors: Sequence[Tuple], world: int, align_bytes: int = 16, min_itemsize: int = 1,
                   tensor_align_elems: int = 0) -> int:
    """tensors: (rows, cols, block_mode[, g_explicit]) per tensor.  Returns the plan handle."""
    out = _P()
    _check(_lib.rs_plan_create(_descs(tensors), len(tensors), int(world), int(align_bytes),
                               int(min_itemsize), int(tensor_align_elems), C.byref(out)),
           "rs_plan_create")
    return out.value


def rs_plan_create_ordered(tensors: Sequence[Tuple], world: int, align_bytes: int = 16,
                           min_itemsize: int = 1, tensor_align_elems: int = 0,
                           order: int = RS_ORDER_DEFAULT) -> int:
    out = _P()
    _check(_lib.rs_plan_create_ordered(_descs(tensors), len(tensors), int(world), int(align_bytes),
                                       int(min_itemsize), int(tensor_align_elems), int(order),
                                       C.byref(out)), "rs_plan_create_ordered")
    return out.value


def rs_plan_create_rooted(tensors: Sequence[Tuple], world: int, roots: Sequence[int],
                          align_bytes: int = 16, min_itemsize: int = 1,
                          tensor_align_elems: int = 0) -> int:
    if len(roots) != len(tensors):
        raise ValueError("one root per tensor")
    out = _P()
    arr = (C.c_int32 * max(1, len(roots)))(*[int(r) for r in roots])
    _check(_lib.rs_plan_create_rooted(_descs(tensors), len(tensors), int(world), int(align_bytes),
                                      int(min_itemsize), int(tensor_align_elems), arr, C.byref(out)),
           "rs_plan_create_rooted")
    return out.value


def rs_select_roots(tensors: Sequence[Tuple], world: int) -> Tuple[List[int], List[float]]:
    """(root of every tensor, accumulated cost of every device)."""
    roots = (C.c_int32 * max(1, len(tensors)))()
    loads = (C.c_double * max(1, int(world)))()
    _check(_lib.rs_select_roots(_descs(tensors), len(tensors), int(world), roots, loads),
           "rs_select_roots")
    return list(roots)[:len(tensors)], list(loads)[:max(0, int(world))]


def rs_shard_dim_granularity(shape: Sequence[int], dim: int, g_user: int) -> int:
    arr = (C.c_int64 * max(1, len(shape)))(*[int(d) for d in shape])
    out = C.c_int64()
    _check(_lib.rs_shard_dim_granularity(arr, len(shape), int(dim), int(g_user), C.byref(out)),
           "rs_shard_dim_granularity")
    return out.value


def rs_plan_order(plan) -> List[int]:
    n = rs_plan_num_tensors(plan)
    out = (C.c_int32 * n)()
    _check(_lib.rs_plan_order(plan, out, n), "rs_plan_order")
    return list(out)


def rs_plan_destroy(plan: int) -> None:
    _lib.rs_plan_destroy(plan)


def rs_check_valid_shard(tensors, world, align_bytes, min_itemsize, tensor_align_elems, S) -> bool:
    return bool(_check(_lib.rs_check_valid_shard(_descs(tensors), len(tensors), int(world),
                                                 int(align_bytes), int(min_itemsize),
                                                 int(tensor_align_elems), int(S)),
                       "rs_check_valid_shard"))


def rs_plan_num_tensors(plan) -> int:
    return _check(_lib.rs_plan_num_tensors(plan), "rs_plan_num_tensors")


def rs_plan_world(plan) -> int:
    return _check(_lib.rs_plan_world(plan), "rs_plan_world")


def rs_plan_shard_elems(plan) -> int:
    return _check(_lib.rs_plan_shard_elems(plan), "rs_plan_shard_elems")


def rs_plan_total_elems(plan) -> int:
    return _check(_lib.rs_plan_total_elems(plan), "rs_plan_total_elems")


def rs_plan_payload_elems(plan) -> int:
    return _check(_lib.rs_plan_payload_elems(plan), "rs_plan_payload_elems")


def rs_plan_padding_elems(plan) -> int:
    return _check(_lib.rs_plan_padding_elems(plan), "rs_plan_padding_elems")


def rs_plan_num_scales(plan) -> int:
    return _check(_lib.rs_plan_num_scales(plan), "rs_plan_num_scales")


def rs_plan_offsets(plan) -> List[int]:
    n = rs_plan_num_tensors(plan)
    out = (C.c_int64 * n)()
    _check(_lib.rs_plan_offsets(plan, out, n), "rs_plan_offsets")
    return list(out)


def rs_plan_scale_bases(plan) -> List[int]:
    n = rs_plan_num_tensors(plan)
    out = (C.c_int64 * (n + 1))()
    _check(_lib.rs_plan_scale_bases(plan, out, n + 1), "rs_plan_scale_bases")
    return list(out)


def rs_plan_scale_range(plan, rank: int) -> Tuple[int, int]:
    lo, hi = C.c_int64(), C.c_int64()
    _check(_lib.rs_plan_scale_range(plan, int(rank), C.byref(lo), C.byref(hi)), "rs_plan_scale_range")
    return lo.value, hi.value


def rs_plan_rank_segments(plan, rank: int) -> List[Tuple[int, int, int, int]]:
    cnt = _check(_lib.rs_plan_rank_segments(plan, int(rank), None, 0), "rs_plan_rank_segments")
    buf = (rs_segment * max(1, cnt))()
    _check(_lib.rs_plan_rank_segments(plan, int(rank), buf, cnt), "rs_plan_rank_segments")
    return [(s.tensor, s.src_off, s.dst_off, s.n) for s in buf[:cnt]]


def rs_plan_upload(plan, device: int = 0) -> None:
    _check(_lib.rs_plan_upload(plan, int(device)), "rs_plan_upload")


def rs_tensor_table_create(plan, tensors: Sequence) -> int:
    """tensors: torch device tensors (contiguous) or raw device addresses, one per plan tensor."""
    n = len(tensors)
    arr = (_P * max(1, n))()
    for i, t in enumerate(tensors):
        if hasattr(t, "is_contiguous") and not t.is_contiguous():
            raise ValueError("tensor table entries must be contiguous")
        arr[i] = _ptr(t)
    if n != rs_plan_num_tensors(plan):
        raise ValueError("one pointer per plan tensor is required")
    out = _P()
    _check(_lib.rs_tensor_table_create(plan, arr, C.byref(out)), "rs_tensor_table_create")
    return out.value


def rs_tensor_table_destroy(table) -> None:
    _lib.rs_tensor_table_destroy(table)


def rs_pack(plan, src_table, dbuf, stream=None) -> None:
    _check(_lib.rs_pack(plan, src_table, _ptr(dbuf), _stream(stream)), "rs_pack")


def rs_pack_noalloc(plan, src_tensors: Sequence, dbuf, stream=None) -> None:
    """src_tensors: torch device tensors (contiguous) or raw device addresses, one per plan tensor."""
    n = len(src_tensors)
    if n != rs_plan_num_tensors(plan):
        raise ValueError("one pointer per plan tensor is required")
    arr = (_P * max(1, n))()
    for i, t in enumerate(src_tensors):
        if hasattr(t, "is_contiguous") and not t.is_contiguous():
            raise ValueError("source tensors must be contiguous")
        arr[i] = _ptr(t)
    _check(_lib.rs_pack_noalloc(plan, arr, _ptr(dbuf), _stream(stream)), "rs_pack_noalloc")


def rs_unpack_bf16(plan, dbuf, dst_table, stream=None) -> None:
    _check(_lib.rs_unpack_bf16(plan, _ptr(dbuf), dst_table, _stream(stream)), "rs_unpack_bf16")


def rs_pack_strided(plan, src_table, dbuf, region_stride: int, stream=None) -> None:
    _check(_lib.rs_pack_strided(plan, src_table, _ptr(dbuf), int(region_stride), _stream(stream)), "rs_pack_strided")


def rs_unpack_bf16_strided(plan, dbuf, region_stride: int, dst_table, stream=None) -> None:
    _check(_lib.rs_unpack_bf16_strided(plan, _ptr(dbuf), int(region_stride), dst_table, _stream(stream)),
           "rs_unpack_bf16_strided")


def rs_pack_scaled(plan, src_table, alpha: float, dbuf, stream=None) -> None:
    _check(_lib.rs_pack_scaled(plan, src_table, float(alpha), _ptr(dbuf), _stream(stream)), "rs_pack_scaled")


def rs_group_add(plan, src_table, alpha: float, dbuf, stream=None) -> None:
    _check(_lib.rs_group_add(plan, src_table, float(alpha), _ptr(dbuf), _stream(stream)), "rs_group_add")


def rs_group_scale(plan, alpha: float, dbuf, stream=None) -> None:
    _check(_lib.rs_group_scale(plan, float(alpha), _ptr(dbuf), _stream(stream)), "rs_group_scale")


def rs_group_zero(plan, dbuf, stream=None) -> None:
    _check(_lib.rs_group_zero(plan, _ptr(dbuf), _stream(stream)), "rs_group_zero")


def rs_reduce(plan, rank: int, partials, row_stride: int, out, stream=None) -> None:
    _check(_lib.rs_reduce(plan, int(rank), _ptr(partials), int(row_stride), _ptr(out), _stream(stream)),
           "rs_reduce")


def rs_reduce_rows(plan, rank: int, partials, rows: int, row_stride: int, out, stream=None) -> None:
    _check(_lib.rs_reduce_rows(plan, int(rank), _ptr(partials), int(rows), int(row_stride), _ptr(out),
                               _stream(stream)), "rs_reduce_rows")


def rs_partials_batch_create(plan, rank: int, partials: Sequence, row_stride: int, outs: Sequence) -> int:
    """partials / outs: one device tensor (or address) per unit, as rs_reduce takes them."""
    n = len(partials)
    if len(outs) != n:
        raise ValueError("one partial buffer and one output per unit")
    a, b = (_P * max(1, n))(), (_P * max(1, n))()
    for i in range(n):
        a[i], b[i] = _ptr(partials[i]), _ptr(outs[i])
    out = _P()
    _check(_lib.rs_partials_batch_create(plan, int(rank), n, a, int(row_stride), b, C.byref(out)),
           "rs_partials_batch_create")
    return out.value


def rs_partials_batch_destroy(batch) -> None:
    _lib.rs_partials_batch_destroy(batch)


def rs_reduce_batch(plan, batch, stream=None) -> None:
    _check(_lib.rs_reduce_batch(plan, batch, _stream(stream)), "rs_reduce_batch")


def rs_quantize(plan, rank: int, shard, codes, scales, stream=None) -> None:
    _check(_lib.rs_quantize(plan, int(rank), _ptr(shard), _ptr(codes), _ptr(scales), _stream(stream)),
           "rs_quantize")


def rs_reduce_quantize(plan, rank: int, partials, row_stride: int, codes, scales, mean_out=None,
                       stream=None) -> None:
    _check(_lib.rs_reduce_quantize(plan, int(rank), _ptr(partials), int(row_stride), _ptr(codes),
                                   _ptr(scales), None if mean_out is None else _ptr(mean_out),
                                   _stream(stream)), "rs_reduce_quantize")


def rs_reduce_quantize_batch(plan, partials_batch, shard_batch, write_means: bool = False, stream=None) -> None:
    _check(_lib.rs_reduce_quantize_batch(plan, partials_batch, shard_batch, int(bool(write_means)),
                                         _stream(stream)), "rs_reduce_quantize_batch")


def rs_shard_batch_create(plan, rank: int, shards: Sequence, codes: Sequence, scales: Sequence) -> int:
    """shards / codes / scales: one device tensor (or address) per unit, as rs_quantize takes them."""
    n = len(shards)
    if not (len(codes) == len(scales) == n):
        raise ValueError("one shard, code buffer and scale slice per unit")
    arrs = []
    for seq in (shards, codes, scales):
        a = (_P * max(1, n))()
        for i, t in enumerate(seq):
            a[i] = _ptr(t)
        arrs.append(a)
    out = _P()
    _check(_lib.rs_shard_batch_create(plan, int(rank), n, arrs[0], arrs[1], arrs[2], C.byref(out)),
           "rs_shard_batch_create")
    return out.value


def rs_shard_batch_destroy(batch) -> None:
    _lib.rs_shard_batch_destroy(batch)


def rs_quantize_batch(plan, batch, stream=None) -> None:
    _check(_lib.rs_quantize_batch(plan, batch, _stream(stream)), "rs_quantize_batch")


def rs_unpack(plan, codes, scales, dst_table, stream=None) -> None:
    _check(_lib.rs_unpack(plan, _ptr(codes), _ptr(scales), dst_table, _stream(stream)), "rs_unpack")


def rs_plan_num_state_blocks(plan) -> int:
    return _check(_lib.rs_plan_num_state_blocks(plan), "rs_plan_num_state_blocks")


def rs_plan_state_bases(plan) -> List[int]:
    n = rs_plan_num_tensors(plan)
    out = (C.c_int64 * (n + 1))()
    _check(_lib.rs_plan_state_bases(plan, out, n + 1), "rs_plan_state_bases")
    return list(out)


def rs_plan_state_range(plan, rank: int) -> Tuple[int, int]:
    lo, hi = C.c_int64(), C.c_int64()
    _check(_lib.rs_plan_state_range(plan, int(rank), C.byref(lo), C.byref(hi)), "rs_plan_state_range")
    return lo.value, hi.value


def rs_state_quantize(plan, rank: int, src, is_unsigned: bool, codes, absmax, stream=None) -> None:
    _check(_lib.rs_state_quantize(plan, int(rank), _ptr(src), int(bool(is_unsigned)), _ptr(codes), _ptr(absmax),
                                  _stream(stream)), "rs_state_quantize")


def rs_state_dequantize(plan, rank: int, codes, absmax, is_unsigned: bool, dst, stream=None) -> None:
    _check(_lib.rs_state_dequantize(plan, int(rank), _ptr(codes), _ptr(absmax), int(bool(is_unsigned)), _ptr(dst),
                                    _stream(stream)), "rs_state_dequantize")


def _hyper(hyper) -> rs_adam8_hyper:
    if isinstance(hyper, rs_adam8_hyper):
        return hyper
    return rs_adam8_hyper(float(hyper[0]), float(hyper[1]), float(hyper[2]), float(hyper[3]), float(hyper[4]),
                          int(hyper[5]))


def rs_adam8_batch_create(plan, rank: int, grads, masters, params_bf16, m_codes, v_codes, m_absmax, v_absmax) -> int:
    """One device tensor (or address) per unit in every sequence; params_bf16 may be None."""
    n = len(grads)
    seqs = [grads, masters, params_bf16, m_codes, v_codes, m_absmax, v_absmax]
    arrs = []
    for seq in seqs:
        if seq is None:
            arrs.append(None)
            continue
        if len(seq) != n:
            raise ValueError("one buffer of every kind per unit")
        a = (_P * max(1, n))()
        for i, t in enumerate(seq):
            a[i] = 0 if t is None else _ptr(t)
        arrs.append(a)
    out = _P()
    _check(_lib.rs_adam8_batch_create(plan, int(rank), n, *arrs, C.byref(out)), "rs_adam8_batch_create")
    return out.value


def rs_adam8_batch_destroy(batch) -> None:
    _lib.rs_adam8_batch_destroy(batch)


def rs_adam8_step_batch(plan, batch, hyper, stream=None) -> None:
    h = _hyper(hyper)
    _check(_lib.rs_adam8_step_batch(plan, batch, C.byref(h), _stream(stream)), "rs_adam8_step_batch")


def rs_adam8_step(plan, rank: int, hyper, grad, master, param_bf16, m_codes, v_codes, m_absmax, v_absmax,
                  stream=None) -> None:
    """hyper: (lr, beta1, beta2, eps, weight_decay, step) or an rs_adam8_hyper; param_bf16 may be None."""
    h = _hyper(hyper)
    _check(_lib.rs_adam8_step(plan, int(rank), C.byref(h), _ptr(grad), _ptr(master),
                              0 if param_bf16 is None else _ptr(param_bf16), _ptr(m_codes), _ptr(v_codes),
                              _ptr(m_absmax), _ptr(v_absmax), _stream(stream)), "rs_adam8_step")


def rs_unpack_f32(plan, codes, scales, dst_table, stream=None) -> None:
    _check(_lib.rs_unpack_f32(plan, _ptr(codes), _ptr(scales), dst_table, _stream(stream)), "rs_unpack_f32")


def rs_unpack_strided(plan, codes, region_stride: int, scales, dst_table, stream=None) -> None:
    _check(_lib.rs_unpack_strided(plan, _ptr(codes), int(region_stride), _ptr(scales), dst_table, _stream(stream)),
           "rs_unpack_strided")


def rs_unpack_f32_strided(plan, codes, region_stride: int, scales, dst_table, stream=None) -> None:
    _check(_lib.rs_unpack_f32_strided(plan, _ptr(codes), int(region_stride), _ptr(scales), dst_table,
                                      _stream(stream)), "rs_unpack_f32_strided")


def rs_copy_probe(dst, src, nbytes: int, stream=None) -> None:
    _check(_lib.rs_copy_probe(_ptr(dst), _ptr(src), int(nbytes), _stream(stream)), "rs_copy_probe")


def raw_call(name: str, *args) -> int:
    """Call an entry point with raw ctypes arguments and get the raw return code (error-path tests)."""
    return getattr(_lib, name)(*args)
