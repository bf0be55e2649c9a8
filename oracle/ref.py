"""ctypes wrapper of the CPU oracle (oracle/slicer_ref.c).  TEST INFRASTRUCTURE ONLY.

numpy arrays in, numpy arrays out; bf16 tensors are uint16 bit patterns.
"""
from __future__ import annotations

import ctypes as C
import os
import numpy as np

from . import build as _build

_DT = {"f32": 0, "bf16": 1}
_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = C.CDLL(path)
        L.slicer_ref_sizes.restype = C.c_int
        L.slicer_ref_sizes.argtypes = [C.c_int, C.c_int64, C.c_int64, C.c_double, C.c_int, C.c_uint32,
                                       C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.slicer_ref_encode.restype = C.c_int
        L.slicer_ref_encode.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_double, C.c_int,
                                        C.c_uint32, C.c_double, C.c_void_p, C.c_void_p, C.c_int]
        L.slicer_ref_encode_ladder.restype = C.c_int
        L.slicer_ref_encode_ladder.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_double, C.c_int,
                                               C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
        L.slicer_ref_sizes_pn.restype = C.c_int
        L.slicer_ref_sizes_pn.argtypes = [C.c_int, C.c_int64, C.c_int64, C.c_double, C.c_int, C.c_int, C.c_uint32,
                                          C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.slicer_ref_encode_pn.restype = C.c_int
        L.slicer_ref_encode_pn.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_double, C.c_int, C.c_int,
                                           C.c_uint32, C.c_double, C.c_void_p, C.c_void_p, C.c_int]
        L.slicer_ref_encode_ds.restype = C.c_int
        L.slicer_ref_encode_ds.argtypes = L.slicer_ref_encode.argtypes
        L.slicer_ref_sizes_csr.restype = C.c_int
        L.slicer_ref_sizes_csr.argtypes = [C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_double, C.c_int, C.c_uint32,
                                           C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
        L.slicer_ref_encode_csr.restype = C.c_int
        L.slicer_ref_encode_csr.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_double, C.c_int,
                                            C.c_uint32, C.c_double, C.c_void_p, C.c_void_p, C.c_int]
        L.slicer_ref_bound.restype = C.c_int
        L.slicer_ref_bound.argtypes = [C.c_int, C.c_int64, C.c_int64, C.c_double, C.c_int, C.c_uint32,
                                       C.POINTER(C.c_uint64), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64)]
        L.slicer_ref_decode.restype = C.c_int
        L.slicer_ref_decode.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int]
        L.slicer_ref_analyze_row.restype = C.c_int
        L.slicer_ref_analyze_row.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_double, C.c_int, C.c_uint32,
                                             C.c_double] + [C.c_void_p] * 8
        L.slicer_ref_encode_atkf.restype = C.c_int
        L.slicer_ref_encode_atkf.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_int64, C.c_double, C.c_double, C.c_int,
                                             C.c_int, C.c_uint32, C.c_double, C.c_void_p, C.c_void_p, C.c_int]
        L.slicer_ref_analyze_row_atkf.restype = C.c_int
        L.slicer_ref_analyze_row_atkf.argtypes = [C.c_void_p, C.c_int, C.c_int64, C.c_double, C.c_double, C.c_int,
                                                  C.c_uint32, C.c_double] + [C.c_void_p] * 5
        _lib = L
    return _lib


def _check_x(x: np.ndarray, dtype: str) -> np.ndarray:
    want = np.float32 if dtype == "f32" else np.uint16
    if x.dtype != want:
        raise TypeError(f"dtype {dtype} needs a {want} array, got {x.dtype}")
    if x.ndim != 2:
        raise ValueError("x must be [rows, row_len]")
    return np.ascontiguousarray(x)


def sizes(dtype: str, rows: int, row_len: int, keep_ratio: float, n_blocks: int, bit_set: int):
    a, b = C.c_size_t(0), C.c_size_t(0)
    rc = lib().slicer_ref_sizes(_DT[dtype], rows, row_len, keep_ratio, n_blocks, bit_set, C.byref(a), C.byref(b))
    if rc:
        raise ValueError(f"slicer_ref_sizes: error {rc}")
    return a.value, b.value


def encode(x: np.ndarray, dtype: str, keep_ratio: float, n_blocks: int, bit_set: int, budget: float,
           n_threads: int = 1):
    """Returns (stream uint32[total_words], meta uint8[meta_bytes])."""
    x = _check_x(x, dtype)
    rows, row_len = x.shape
    cap, mb = sizes(dtype, rows, row_len, keep_ratio, n_blocks, bit_set)
    stream = np.zeros(max(cap // 4, 1), np.uint32)
    meta = np.zeros(mb, np.uint8)
    rc = lib().slicer_ref_encode(x.ctypes.data, _DT[dtype], rows, row_len, keep_ratio, n_blocks, bit_set,
                                 budget, stream.ctypes.data, meta.ctypes.data, n_threads)
    if rc:
        raise ValueError(f"slicer_ref_encode: error {rc}")
    total = int(meta[48:56].view(np.uint64)[0])
    return stream[:total].copy(), meta


def encode_pn(x: np.ndarray, dtype: str, keep_ratio: float, n_blocks: int, n_blocks_neg: int, bit_set: int,
              budget: float, n_threads: int = 1):
    """Separate block counts for the positive and the negative class.  Returns (stream, meta)."""
    x = _check_x(x, dtype)
    rows, row_len = x.shape
    a, b = C.c_size_t(0), C.c_size_t(0)
    rc = lib().slicer_ref_sizes_pn(_DT[dtype], rows, row_len, keep_ratio, n_blocks, n_blocks_neg, bit_set,
                                   C.byref(a), C.byref(b))
    if rc:
        raise ValueError(f"slicer_ref_sizes_pn: error {rc}")
    stream = np.zeros(max(a.value // 4, 1), np.uint32)
    meta = np.zeros(b.value, np.uint8)
    rc = lib().slicer_ref_encode_pn(x.ctypes.data, _DT[dtype], rows, row_len, keep_ratio, n_blocks, n_blocks_neg,
                                    bit_set, budget, stream.ctypes.data, meta.ctypes.data, n_threads)
    if rc:
        raise ValueError(f"slicer_ref_encode_pn: error {rc}")
    total = int(meta[48:56].view(np.uint64)[0])
    return stream[:total].copy(), meta


def encode_atkf(x: np.ndarray, dtype: str, keep_ratio: float, lam: float, n_blocks: int, n_blocks_neg: int,
                bit_set: int, budget: float, n_threads: int = 1):
    """Asymmetric thresholds of Sec. 3.1 (lambda in [0, 1)).  Returns (stream, meta)."""
    x = _check_x(x, dtype)
    rows, row_len = x.shape
    a, b = C.c_size_t(0), C.c_size_t(0)
    rc = lib().slicer_ref_sizes_pn(_DT[dtype], rows, row_len, keep_ratio, n_blocks, n_blocks_neg, bit_set,
                                   C.byref(a), C.byref(b))
    if rc:
        raise ValueError(f"slicer_ref_sizes_pn: error {rc}")
    stream = np.zeros(max(a.value // 4, 1), np.uint32)
    meta = np.zeros(b.value, np.uint8)
    rc = lib().slicer_ref_encode_atkf(x.ctypes.data, _DT[dtype], rows, row_len, keep_ratio, lam, n_blocks,
                                      n_blocks_neg, bit_set, budget, stream.ctypes.data, meta.ctypes.data, n_threads)
    if rc:
        raise ValueError(f"slicer_ref_encode_atkf: error {rc}")
    total = int(meta[48:56].view(np.uint64)[0])
    return stream[:total].copy(), meta


def analyze_row_atkf(x_row: np.ndarray, dtype: str, keep_ratio: float, lam: float, n_blocks: int, bit_set: int,
                     budget: float):
    """Per-element view of one row under the asymmetric thresholds (block_of, code_of, vmin, vmax, qb)."""
    x_row = np.ascontiguousarray(x_row)
    N = x_row.shape[0]
    M2 = 2 * n_blocks
    out = dict(block_of=np.empty(N, np.int32), code_of=np.empty(N, np.uint32),
               vmin=np.empty(M2, np.float32), vmax=np.empty(M2, np.float32), qb=np.empty(M2, np.uint8))
    rc = lib().slicer_ref_analyze_row_atkf(x_row.ctypes.data, _DT[dtype], N, keep_ratio, lam, n_blocks, bit_set,
                                           budget, *[out[k].ctypes.data for k in
                                                     ("block_of", "code_of", "vmin", "vmax", "qb")])
    if rc:
        raise ValueError(f"slicer_ref_analyze_row_atkf: error {rc}")
    return out


def encode_ds(x: np.ndarray, dtype: str, keep_ratio: float, n_blocks: int, bit_set: int, delta: float,
              n_threads: int = 1):
    """The paper's DS guard with greedy descent from max(bit_set).  Returns (stream, meta)."""
    x = _check_x(x, dtype)
    rows, row_len = x.shape
    cap, mb = sizes(dtype, rows, row_len, keep_ratio, n_blocks, bit_set)
    stream = np.zeros(max(cap // 4, 1), np.uint32)
    meta = np.zeros(mb, np.uint8)
    rc = lib().slicer_ref_encode_ds(x.ctypes.data, _DT[dtype], rows, row_len, keep_ratio, n_blocks, bit_set,
                                    delta, stream.ctypes.data, meta.ctypes.data, n_threads)
    if rc:
        raise ValueError(f"slicer_ref_encode_ds: error {rc}")
    total = int(meta[48:56].view(np.uint64)[0])
    return stream[:total].copy(), meta


def encode_csr(x: np.ndarray, dtype: str, n_rows: int, n_cols: int, keep_ratio: float, n_blocks: int, bit_set: int,
               budget: float, n_threads: int = 1):
    """Two-dimensional instances: x is [instances, n_rows * n_cols]; blocks are stored as CSR triples.
    Returns (stream, meta)."""
    x = _check_x(x, dtype)
    rows, row_len = x.shape
    if row_len != n_rows * n_cols:
        raise ValueError("row length must be n_rows * n_cols")
    a, b = C.c_size_t(0), C.c_size_t(0)
    rc = lib().slicer_ref_sizes_csr(_DT[dtype], rows, n_rows, n_cols, keep_ratio, n_blocks, bit_set, C.byref(a), C.byref(b))
    if rc:
        raise ValueError(f"slicer_ref_sizes_csr: error {rc}")
    stream = np.zeros(max(a.value // 4, 1), np.uint32)
    meta = np.zeros(b.value, np.uint8)
    rc = lib().slicer_ref_encode_csr(x.ctypes.data, _DT[dtype], rows, n_rows, n_cols, keep_ratio, n_blocks, bit_set,
                                     budget, stream.ctypes.data, meta.ctypes.data, n_threads)
    if rc:
        raise ValueError(f"slicer_ref_encode_csr: error {rc}")
    total = int(meta[48:56].view(np.uint64)[0])
    return stream[:total].copy(), meta


def ladder_bit_set(ladder) -> int:
    bs = 0
    for q in ladder:
        bs |= 1 << int(q)
    return bs


def encode_ladder(x: np.ndarray, dtype: str, keep_ratio: float, ladder, n_threads: int = 1):
    """Fixed multi-level mode: block m of each sign class uses ladder[m] bits (n_blocks = len(ladder))."""
    x = _check_x(x, dtype)
    rows, row_len = x.shape
    lad = np.ascontiguousarray(np.asarray(ladder, np.uint8))
    M = int(lad.size)
    cap, mb = sizes(dtype, rows, row_len, keep_ratio, M, ladder_bit_set(lad))
    stream = np.zeros(max(cap // 4, 1), np.uint32)
    meta = np.zeros(mb, np.uint8)
    rc = lib().slicer_ref_encode_ladder(x.ctypes.data, _DT[dtype], rows, row_len, keep_ratio, M,
                                        lad.ctypes.data, stream.ctypes.data, meta.ctypes.data, n_threads)
    if rc:
        raise ValueError(f"slicer_ref_encode_ladder: error {rc}")
    total = int(meta[48:56].view(np.uint64)[0])
    return stream[:total].copy(), meta


def bound(dtype: str, rows: int, row_len: int, keep_ratio: float, n_blocks: int, bit_set: int):
    """(value_bits, index_bits, header_bits) of the payload's upper bound."""
    v, i, h = C.c_uint64(0), C.c_uint64(0), C.c_uint64(0)
    rc = lib().slicer_ref_bound(_DT[dtype], rows, row_len, keep_ratio, n_blocks, bit_set,
                                C.byref(v), C.byref(i), C.byref(h))
    if rc:
        raise ValueError(f"slicer_ref_bound: error {rc}")
    return v.value, i.value, h.value


def decode(stream: np.ndarray, meta: np.ndarray, n_threads: int = 1) -> np.ndarray:
    """Dense tensor [rows,row_len]: float32, or uint16 bf16 bits."""
    meta = np.ascontiguousarray(meta, np.uint8)
    stream = np.ascontiguousarray(stream, np.uint32)
    if stream.size == 0:
        stream = np.zeros(1, np.uint32)
    dt = int(meta[8:12].view(np.uint32)[0])
    rows = int(meta[16:24].view(np.uint64)[0])
    row_len = int(meta[24:32].view(np.uint64)[0])
    y = np.empty((rows, row_len), np.float32 if dt == 0 else np.uint16)
    rc = lib().slicer_ref_decode(stream.ctypes.data, meta.ctypes.data, y.ctypes.data, n_threads)
    if rc:
        raise ValueError(f"slicer_ref_decode: error {rc}")
    return y


def analyze_row(x_row: np.ndarray, dtype: str, keep_ratio: float, n_blocks: int, bit_set: int, budget: float):
    """Per-element / per-block view of one row before packing (see slicer_ref.h)."""
    x_row = np.ascontiguousarray(x_row)
    N = x_row.shape[0]
    M2 = 2 * n_blocks
    out = dict(block_of=np.empty(N, np.int32), code_of=np.empty(N, np.uint32),
               vmin=np.empty(M2, np.float32), vmax=np.empty(M2, np.float32), qb=np.empty(M2, np.uint8),
               s_int=np.empty((M2, 17), np.uint64), e_int=np.empty(M2, np.uint64), e_exp=np.empty(M2, np.int32))
    rc = lib().slicer_ref_analyze_row(x_row.ctypes.data, _DT[dtype], N, keep_ratio, n_blocks, bit_set, budget,
                                      *[out[k].ctypes.data for k in
                                        ("block_of", "code_of", "vmin", "vmax", "qb", "s_int", "e_int", "e_exp")])
    if rc:
        raise ValueError(f"slicer_ref_analyze_row: error {rc}")
    return out
