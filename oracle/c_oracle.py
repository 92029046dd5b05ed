"""Loader of the C / OpenMP oracle (oracle/c/oracle.c).  TEST INFRASTRUCTURE ONLY.

A second statement of the same definitions as the numpy oracle (pack, reduce in double, FP8
block quantisation and its inverse), written separately in plain C; the tests hold the two
against each other bit for bit, and the bench times it on all host cores."""
from __future__ import annotations

import ctypes as C
import os
import shutil
import subprocess
from typing import Sequence, Tuple

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(HERE, "c", "oracle.c")
LIB = os.path.join(HERE, "c", "liboracle_c.so")


def build(verbose: bool = False) -> str:
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        raise RuntimeError("no C compiler for the C oracle")
    cmd = [cc, "-O2", "-std=c99", "-fopenmp", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math",
           "-Wall", "-Wextra", SRC, "-lm", "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("C oracle failed to build:\n" + res.stderr)
    return LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB) or os.path.getmtime(LIB) < os.path.getmtime(SRC):
            build()
        _lib = C.CDLL(LIB)
        _lib.oc_e4m3_value.restype = C.c_float
        _lib.oc_e4m3_value.argtypes = [C.c_uint8]
        _lib.oc_e4m3_encode.restype = C.c_uint8
        _lib.oc_e4m3_encode.argtypes = [C.c_float]
        _lib.oc_f32_to_bf16.restype = C.c_uint16
        _lib.oc_f32_to_bf16.argtypes = [C.c_float]
        _lib.oc_num_threads.restype = C.c_int
        _lib.oc_set_num_threads.argtypes = [C.c_int]
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(C.c_void_p)


def num_threads() -> int:
    return int(lib().oc_num_threads())


def set_num_threads(n: int) -> None:
    lib().oc_set_num_threads(int(n))


def ragged_pack(srcs: Sequence[np.ndarray], offsets: Sequence[int], total: int) -> np.ndarray:
    flat = [np.ascontiguousarray(s, dtype=np.uint16).reshape(-1) for s in srcs]
    ptrs = (C.c_void_p * len(flat))(*[f.ctypes.data for f in flat])
    offs = np.asarray(offsets, dtype=np.int64)
    sizes = np.asarray([f.size for f in flat], dtype=np.int64)
    db = np.empty(total, dtype=np.uint16)
    lib().oc_ragged_pack(ptrs, _p(offs), _p(sizes), len(flat), _p(db), C.c_int64(total))
    return db


def shard_reduce(partials: np.ndarray, segments: Sequence[Tuple[int, int, int, int]]) -> np.ndarray:
    P = np.ascontiguousarray(partials, dtype=np.uint16)
    W, S = P.shape
    off = np.asarray([s[2] for s in segments], dtype=np.int64)
    ln = np.asarray([s[3] for s in segments], dtype=np.int64)
    out = np.empty(S, dtype=np.float32)
    lib().oc_shard_reduce(_p(P), W, C.c_int64(S), _p(off), _p(ln), len(segments), _p(out))
    return out


def shard_reduce_f32_ordered(partials: np.ndarray, segments: Sequence[Tuple[int, int, int, int]]) -> np.ndarray:
    P = np.ascontiguousarray(partials, dtype=np.uint16)
    W, S = P.shape
    off = np.asarray([s[2] for s in segments], dtype=np.int64)
    ln = np.asarray([s[3] for s in segments], dtype=np.int64)
    out = np.empty(S, dtype=np.float32)
    lib().oc_shard_reduce_f32_ordered(_p(P), W, C.c_int64(S), _p(off), _p(ln), len(segments), _p(out))
    return out


def shard_reduce_abs_sum(partials: np.ndarray) -> np.ndarray:
    P = np.ascontiguousarray(partials, dtype=np.uint16)
    W, S = P.shape
    out = np.empty(S, dtype=np.float64)
    lib().oc_shard_abs_sum(_p(P), W, C.c_int64(S), _p(out))
    return out


def quantise_matrix(bits: np.ndarray, bh: int, bw: int) -> Tuple[np.ndarray, np.ndarray]:
    x = np.ascontiguousarray(bits, dtype=np.uint16)
    R, Cc = x.shape
    codes = np.empty((R, Cc), dtype=np.uint8)
    scales = np.empty((-(-R // bh), -(-Cc // bw)), dtype=np.float32)
    lib().oc_quantise_matrix(_p(x), C.c_int64(R), C.c_int64(Cc), int(bh), int(bw), _p(codes), _p(scales))
    return codes, scales


def dequantise_matrix(codes: np.ndarray, scales: np.ndarray, bh: int, bw: int) -> np.ndarray:
    c = np.ascontiguousarray(codes, dtype=np.uint8)
    s = np.ascontiguousarray(scales, dtype=np.float32)
    R, Cc = c.shape
    out = np.empty((R, Cc), dtype=np.uint16)
    lib().oc_dequantise_matrix(_p(c), _p(s), C.c_int64(R), C.c_int64(Cc), int(bh), int(bw), _p(out))
    return out
