"""Thin Python binding of libslicer.so (include/slicer.h): argument marshalling only.

Every step of the codec runs in the HIP kernels; PyTorch supplies device memory and
the current HIP stream.  There is no CPU fallback: if the library has not been built
(``python -m paper_2511_11608_amd.build``) loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libslicer.so")

SLICER_F32, SLICER_BF16 = 0, 1
_TORCH_DT = {torch.float32: SLICER_F32, torch.bfloat16: SLICER_BF16}

_lib = None


class SlicerError(RuntimeError):
    def __init__(self, fn: str, code: int):
        L = load()
        msg = L.slicer_strerror(code).decode()
        extra = f" (hipError {L.slicer_last_hip_error()})" if code == -3 else ""
        super().__init__(f"{fn}: {msg}{extra} [{code}]")
        self.code = code


def load() -> C.CDLL:
    """Load libslicer.so; fails loudly when it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2511_11608_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i64, dbl, u32, cint = C.c_void_p, C.c_int64, C.c_double, C.c_uint32, C.c_int
        szp = C.POINTER(C.c_size_t)
        L.slicer_sizes.restype = cint
        L.slicer_sizes.argtypes = [cint, i64, i64, dbl, cint, u32, szp, szp, szp]
        L.slicer_encode_path.restype = cint
        L.slicer_encode_path.argtypes = [cint, i64, i64, dbl, cint, u32]
        L.slicer_encode.restype = cint
        L.slicer_encode.argtypes = [vp, cint, i64, i64, dbl, cint, u32, dbl, vp, vp, vp, vp]
        L.slicer_encode_static.restype = cint
        L.slicer_encode_static.argtypes = [vp, cint, i64, i64, dbl, cint, u32, dbl, vp, vp, vp]
        L.slicer_sizes_csr.restype = cint
        L.slicer_sizes_csr.argtypes = [cint, i64, i64, i64, dbl, cint, u32, szp, szp, szp]
        L.slicer_encode_csr.restype = cint
        L.slicer_encode_csr.argtypes = [vp, cint, i64, i64, i64, dbl, cint, u32, dbl, vp, vp, vp, vp]
        L.slicer_decode_as_csr.restype = cint
        L.slicer_decode_as_csr.argtypes = [vp, vp, vp, cint, i64, i64, i64, cint, vp]
        L.slicer_check_csr.restype = cint
        L.slicer_check_csr.argtypes = [vp, C.c_uint64, cint, i64, i64, i64, cint, vp, vp]
        L.slicer_sizes_pn.restype = cint
        L.slicer_sizes_pn.argtypes = [cint, i64, i64, dbl, cint, cint, u32, szp, szp, szp]
        L.slicer_encode_pn.restype = cint
        L.slicer_encode_pn.argtypes = [vp, cint, i64, i64, dbl, cint, cint, u32, dbl, vp, vp, vp, vp]
        L.slicer_encode_atkf.restype = cint
        L.slicer_encode_atkf.argtypes = [vp, cint, i64, i64, dbl, dbl, cint, cint, u32, dbl, vp, vp, vp, vp]
        L.slicer_decode_as_pn.restype = cint
        L.slicer_decode_as_pn.argtypes = [vp, vp, vp, cint, i64, i64, cint, cint, vp]
        L.slicer_check_pn.restype = cint
        L.slicer_check_pn.argtypes = [vp, C.c_uint64, cint, i64, i64, cint, cint, vp, vp]
        L.slicer_encode_ds.restype = cint
        L.slicer_encode_ds.argtypes = L.slicer_encode.argtypes
        L.slicer_encode_ladder.restype = cint
        L.slicer_encode_ladder.argtypes = [vp, cint, i64, i64, dbl, cint, C.c_char_p, vp, vp, vp, vp]
        L.slicer_ladder_bit_set.restype = u32
        L.slicer_ladder_bit_set.argtypes = [C.c_char_p, cint]
        L.slicer_bound.restype = cint
        L.slicer_bound.argtypes = [cint, i64, i64, dbl, cint, u32] + [C.POINTER(C.c_uint64)] * 3
        L.slicer_decode.restype = cint
        L.slicer_decode.argtypes = [vp, vp, vp, vp]
        L.slicer_decode_as.restype = cint
        L.slicer_decode_as.argtypes = [vp, vp, vp, cint, i64, i64, cint, vp]
        L.slicer_check.restype = cint
        L.slicer_check.argtypes = [vp, C.c_uint64, cint, i64, i64, cint, vp, vp]
        L.slicer_stream_words.restype = cint
        L.slicer_stream_words.argtypes = [vp, C.POINTER(C.c_uint64), vp]
        L.slicer_arith_probe.restype = cint
        L.slicer_arith_probe.argtypes = [cint, vp, vp, vp, i64, vp]
        L.slicer_profile_events.restype = cint
        L.slicer_profile_events.argtypes = [vp, vp]
        L.slicer_last_hip_error.restype = cint
        L.slicer_last_hip_error.argtypes = []
        L.slicer_strerror.restype = C.c_char_p
        L.slicer_strerror.argtypes = [cint]
        _lib = L
    return _lib


def _check(fn: str, rc: int) -> None:
    if rc != 0:
        raise SlicerError(fn, rc)


def _stream_handle(stream) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream


def _dt_of(x: torch.Tensor) -> int:
    if x.dtype not in _TORCH_DT:
        raise TypeError(f"unsupported tensor dtype {x.dtype}")
    return _TORCH_DT[x.dtype]


def slicer_sizes(dt: int, rows: int, row_len: int, keep_ratio: float, n_blocks: int, bit_set: int):
    """(stream_capacity_bytes, meta_bytes, workspace_bytes) for one encode call."""
    a, b, c = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    _check("slicer_sizes", load().slicer_sizes(dt, rows, row_len, keep_ratio, n_blocks, bit_set,
                                               C.byref(a), C.byref(b), C.byref(c)))
    return a.value, b.value, c.value


def slicer_encode_path(dt: int, rows: int, row_len: int, keep_ratio: float, n_blocks: int, bit_set: int) -> int:
    """0 generic, 1 row-resident, 2 long-row kernel family for this shape."""
    rc = load().slicer_encode_path(dt, rows, row_len, keep_ratio, n_blocks, bit_set)
    if rc < 0:
        raise SlicerError("slicer_encode_path", rc)
    return rc


def alloc_buffers(x: torch.Tensor, keep_ratio: float, n_blocks: int, bit_set: int):
    """Device buffers (stream int32, meta uint8, workspace uint8) sized for x [rows,row_len]."""
    rows, row_len = x.shape
    cap, mb, wb = slicer_sizes(_dt_of(x), rows, row_len, keep_ratio, n_blocks, bit_set)
    dev = x.device
    return (torch.empty(max(cap // 4, 1), dtype=torch.int32, device=dev),
            torch.empty(mb, dtype=torch.uint8, device=dev),
            torch.empty(max(wb, 256), dtype=torch.uint8, device=dev))


def slicer_encode(x: torch.Tensor, keep_ratio: float, n_blocks: int, bit_set: int, distortion_budget: float,
                  stream_buf: torch.Tensor, meta: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    """Enqueue the encode of x [rows,row_len] (fp32 or bf16, contiguous, on the GPU)."""
    if not x.is_cuda or not x.is_contiguous() or x.dim() != 2:
        raise ValueError("x must be a contiguous 2-D tensor on the GPU")
    rows, row_len = x.shape
    _check("slicer_encode", load().slicer_encode(
        x.data_ptr(), _dt_of(x), rows, row_len, keep_ratio, n_blocks, bit_set, distortion_budget,
        stream_buf.data_ptr(), meta.data_ptr(), workspace.data_ptr(), _stream_handle(stream)))


def slicer_encode_static(x: torch.Tensor, keep_ratio: float, n_blocks: int, bit_set: int, distortion_budget: float,
                         stream_buf: torch.Tensor, meta: torch.Tensor, stream=None) -> None:
    """slicer_encode on the library's static scratch: no workspace argument, nothing allocated."""
    if not x.is_cuda or not x.is_contiguous() or x.dim() != 2:
        raise ValueError("x must be a contiguous 2-D tensor on the GPU")
    rows, row_len = x.shape
    _check("slicer_encode_static", load().slicer_encode_static(
        x.data_ptr(), _dt_of(x), rows, row_len, keep_ratio, n_blocks, bit_set, distortion_budget,
        stream_buf.data_ptr(), meta.data_ptr(), _stream_handle(stream)))


def alloc_buffers_csr(x: torch.Tensor, n_rows: int, n_cols: int, keep_ratio: float, n_blocks: int, bit_set: int):
    """Device buffers for two-dimensional instances: x is [instances, n_rows * n_cols]."""
    a, b, c = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    _check("slicer_sizes_csr", load().slicer_sizes_csr(_dt_of(x), x.shape[0], n_rows, n_cols, keep_ratio, n_blocks,
                                                      bit_set, C.byref(a), C.byref(b), C.byref(c)))
    dev = x.device
    return (torch.empty(max(a.value // 4, 1), dtype=torch.int32, device=dev),
            torch.empty(b.value, dtype=torch.uint8, device=dev),
            torch.empty(max(c.value, 256), dtype=torch.uint8, device=dev))


def slicer_encode_csr(x: torch.Tensor, n_rows: int, n_cols: int, keep_ratio: float, n_blocks: int, bit_set: int,
                      distortion_budget: float, stream_buf: torch.Tensor, meta: torch.Tensor, workspace: torch.Tensor,
                      stream=None) -> None:
    """Encode instances of n_rows x n_cols with every block stored as CSR(values, columns, row pointers)."""
    if not x.is_cuda or not x.is_contiguous() or x.dim() != 2 or x.shape[1] != n_rows * n_cols:
        raise ValueError("x must be a contiguous [instances, n_rows * n_cols] tensor on the GPU")
    _check("slicer_encode_csr", load().slicer_encode_csr(
        x.data_ptr(), _dt_of(x), x.shape[0], n_rows, n_cols, keep_ratio, n_blocks, bit_set, distortion_budget,
        stream_buf.data_ptr(), meta.data_ptr(), workspace.data_ptr(), _stream_handle(stream)))


def slicer_decode_as_csr(stream_buf: torch.Tensor, meta: torch.Tensor, y: torch.Tensor, n_rows: int, n_cols: int,
                         n_blocks: int, stream=None) -> None:
    _check("slicer_decode_as_csr", load().slicer_decode_as_csr(stream_buf.data_ptr(), meta.data_ptr(), y.data_ptr(),
                                                              _dt_of(y), y.shape[0], n_rows, n_cols, n_blocks,
                                                              _stream_handle(stream)))


def slicer_check_csr(meta: torch.Tensor, stream_words: int, y_like: torch.Tensor, n_rows: int, n_cols: int, n_blocks: int,
                     stream=None) -> None:
    """Validate a received meta buffer of two-dimensional instances; raises SlicerError (-4)."""
    scratch = torch.empty(64, dtype=torch.int32, device=meta.device)
    _check("slicer_check_csr", load().slicer_check_csr(meta.data_ptr(), stream_words, _dt_of(y_like), y_like.shape[0],
                                                      n_rows, n_cols, n_blocks, scratch.data_ptr(), _stream_handle(stream)))


def alloc_buffers_pn(x: torch.Tensor, keep_ratio: float, n_blocks: int, n_blocks_neg: int, bit_set: int):
    """Device buffers for separate block counts of the two sign classes."""
    rows, row_len = x.shape
    a, b, c = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
    _check("slicer_sizes_pn", load().slicer_sizes_pn(_dt_of(x), rows, row_len, keep_ratio, n_blocks, n_blocks_neg,
                                                    bit_set, C.byref(a), C.byref(b), C.byref(c)))
    dev = x.device
    return (torch.empty(max(a.value // 4, 1), dtype=torch.int32, device=dev),
            torch.empty(b.value, dtype=torch.uint8, device=dev),
            torch.empty(max(c.value, 256), dtype=torch.uint8, device=dev))


def slicer_encode_pn(x: torch.Tensor, keep_ratio: float, n_blocks: int, n_blocks_neg: int, bit_set: int,
                     distortion_budget: float, stream_buf: torch.Tensor, meta: torch.Tensor, workspace: torch.Tensor,
                     stream=None) -> None:
    """slicer_encode with n_blocks blocks for the positive and n_blocks_neg for the negative class."""
    if not x.is_cuda or not x.is_contiguous() or x.dim() != 2:
        raise ValueError("x must be a contiguous 2-D tensor on the GPU")
    rows, row_len = x.shape
    _check("slicer_encode_pn", load().slicer_encode_pn(
        x.data_ptr(), _dt_of(x), rows, row_len, keep_ratio, n_blocks, n_blocks_neg, bit_set, distortion_budget,
        stream_buf.data_ptr(), meta.data_ptr(), workspace.data_ptr(), _stream_handle(stream)))


def slicer_encode_atkf(x: torch.Tensor, keep_ratio: float, lam: float, n_blocks: int, n_blocks_neg: int, bit_set: int,
                       distortion_budget: float, stream_buf: torch.Tensor, meta: torch.Tensor, workspace: torch.Tensor,
                       stream=None) -> None:
    """slicer_encode_pn with the asymmetric thresholds of Sec. 3.1 (asymmetry factor lam in [0, 1))."""
    if not x.is_cuda or not x.is_contiguous() or x.dim() != 2:
        raise ValueError("x must be a contiguous 2-D tensor on the GPU")
    rows, row_len = x.shape
    _check("slicer_encode_atkf", load().slicer_encode_atkf(
        x.data_ptr(), _dt_of(x), rows, row_len, keep_ratio, lam, n_blocks, n_blocks_neg, bit_set, distortion_budget,
        stream_buf.data_ptr(), meta.data_ptr(), workspace.data_ptr(), _stream_handle(stream)))


def slicer_decode_as_pn(stream_buf: torch.Tensor, meta: torch.Tensor, y: torch.Tensor, n_blocks: int,
                        n_blocks_neg: int, stream=None) -> None:
    rows, row_len = y.shape
    _check("slicer_decode_as_pn", load().slicer_decode_as_pn(stream_buf.data_ptr(), meta.data_ptr(), y.data_ptr(),
                                                            _dt_of(y), rows, row_len, n_blocks, n_blocks_neg,
                                                            _stream_handle(stream)))


def slicer_check_pn(meta: torch.Tensor, stream_words: int, y_like: torch.Tensor, n_blocks: int, n_blocks_neg: int,
                    stream=None) -> None:
    rows, row_len = y_like.shape
    scratch = torch.empty(64, dtype=torch.int32, device=meta.device)
    _check("slicer_check_pn", load().slicer_check_pn(meta.data_ptr(), stream_words, _dt_of(y_like), rows, row_len,
                                                    n_blocks, n_blocks_neg, scratch.data_ptr(), _stream_handle(stream)))


def slicer_encode_ds(x: torch.Tensor, keep_ratio: float, n_blocks: int, bit_set: int, delta: float,
                     stream_buf: torch.Tensor, meta: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    """Encode with the DS guard of Sec. 3.2.1 (greedy descent from max(bit_set) while DS <= delta)."""
    if not x.is_cuda or not x.is_contiguous() or x.dim() != 2:
        raise ValueError("x must be a contiguous 2-D tensor on the GPU")
    rows, row_len = x.shape
    _check("slicer_encode_ds", load().slicer_encode_ds(
        x.data_ptr(), _dt_of(x), rows, row_len, keep_ratio, n_blocks, bit_set, delta,
        stream_buf.data_ptr(), meta.data_ptr(), workspace.data_ptr(), _stream_handle(stream)))


def slicer_ladder_bit_set(ladder) -> int:
    """Set of the ladder's bitwidths (0 if an entry is outside 1..16)."""
    lad = bytes(int(q) & 0xFF for q in ladder)
    return load().slicer_ladder_bit_set(lad, len(lad))


def slicer_encode_ladder(x: torch.Tensor, keep_ratio: float, ladder, stream_buf: torch.Tensor, meta: torch.Tensor,
                         workspace: torch.Tensor, stream=None) -> None:
    """Fixed multi-level mode: block m of each sign class uses ladder[m] bits (n_blocks = len(ladder))."""
    if not x.is_cuda or not x.is_contiguous() or x.dim() != 2:
        raise ValueError("x must be a contiguous 2-D tensor on the GPU")
    rows, row_len = x.shape
    lad = bytes(int(q) & 0xFF for q in ladder)
    _check("slicer_encode_ladder", load().slicer_encode_ladder(
        x.data_ptr(), _dt_of(x), rows, row_len, keep_ratio, len(lad), lad,
        stream_buf.data_ptr(), meta.data_ptr(), workspace.data_ptr(), _stream_handle(stream)))


def slicer_bound(dt: int, rows: int, row_len: int, keep_ratio: float, n_blocks: int, bit_set: int):
    """(value_bits, index_bits, header_bits) of the payload's upper bound; host computation."""
    v, i, h = C.c_uint64(0), C.c_uint64(0), C.c_uint64(0)
    _check("slicer_bound", load().slicer_bound(dt, rows, row_len, keep_ratio, n_blocks, bit_set,
                                               C.byref(v), C.byref(i), C.byref(h)))
    return v.value, i.value, h.value


def slicer_check(meta: torch.Tensor, stream_words: int, y_like: torch.Tensor, n_blocks: int, stream=None) -> None:
    """Validate a received meta buffer against the shape of y_like and the words held; raises SlicerError (-4)."""
    rows, row_len = y_like.shape
    scratch = torch.empty(64, dtype=torch.int32, device=meta.device)
    _check("slicer_check", load().slicer_check(meta.data_ptr(), stream_words, _dt_of(y_like), rows, row_len, n_blocks,
                                              scratch.data_ptr(), _stream_handle(stream)))


def slicer_decode(stream_buf: torch.Tensor, meta: torch.Tensor, y: torch.Tensor, stream=None) -> None:
    """Decode into y using the header stored in meta (reads it to the host, waits for the stream)."""
    _check("slicer_decode", load().slicer_decode(stream_buf.data_ptr(), meta.data_ptr(), y.data_ptr(),
                                                 _stream_handle(stream)))


def slicer_decode_as(stream_buf: torch.Tensor, meta: torch.Tensor, y: torch.Tensor, n_blocks: int,
                     stream=None) -> None:
    """Decode into y [rows,row_len] with the shape taken from y; asynchronous."""
    if not y.is_cuda or not y.is_contiguous() or y.dim() != 2:
        raise ValueError("y must be a contiguous 2-D tensor on the GPU")
    rows, row_len = y.shape
    _check("slicer_decode_as", load().slicer_decode_as(stream_buf.data_ptr(), meta.data_ptr(), y.data_ptr(),
                                                       _dt_of(y), rows, row_len, n_blocks,
                                                       _stream_handle(stream)))


def slicer_stream_words(meta: torch.Tensor, stream=None) -> int:
    """Number of 32-bit stream words the last encode into `meta` produced (waits for the stream)."""
    w = C.c_uint64(0)
    _check("slicer_stream_words", load().slicer_stream_words(meta.data_ptr(), C.byref(w), _stream_handle(stream)))
    return w.value


def slicer_arith_probe(op: int, a: torch.Tensor, b: torch.Tensor, out: torch.Tensor, stream=None) -> None:
    """One elementary operation of the codec's arithmetic on int32 tensors of fp32 bit patterns (see slicer.h)."""
    _check("slicer_arith_probe", load().slicer_arith_probe(op, a.data_ptr(), b.data_ptr(), out.data_ptr(), a.numel(),
                                                          _stream_handle(stream)))


def slicer_profile_events(start_event, stop_event) -> None:
    """Raw hipEvent_t handles (ints) or None, None: see include/slicer.h."""
    _check("slicer_profile_events", load().slicer_profile_events(start_event, stop_event))
