"""Helpers for the GPU parity tests: run a workload through the HIP library via its
C ABI and bring stream / meta / decoded tensor back as numpy arrays."""
from __future__ import annotations

import numpy as np
import torch

from paper_2511_11608_amd import binding
from paper_2511_11608_amd.devmem import to_device, to_host  # noqa: F401 (re-exported for the tests)


def gpu_encode(x: np.ndarray, dtype: str, keep_ratio, n_blocks, bit_set, budget):
    xd = to_device(x, dtype)
    sb, meta, ws = binding.alloc_buffers(xd, keep_ratio, n_blocks, bit_set)
    ws.fill_(0xA5)          # the encoder must not rely on workspace contents
    sb.fill_(-1)
    meta.fill_(0xFF)
    binding.slicer_encode(xd, keep_ratio, n_blocks, bit_set, budget, sb, meta, ws)
    words = binding.slicer_stream_words(meta)
    return sb, meta, words


def gpu_encode_ds(x: np.ndarray, dtype: str, keep_ratio, n_blocks, bit_set, delta):
    xd = to_device(x, dtype)
    sb, meta, ws = binding.alloc_buffers(xd, keep_ratio, n_blocks, bit_set)
    ws.fill_(0xA5)
    sb.fill_(-1)
    meta.fill_(0xFF)
    binding.slicer_encode_ds(xd, keep_ratio, n_blocks, bit_set, delta, sb, meta, ws)
    words = binding.slicer_stream_words(meta)
    return sb, meta, words


def gpu_encode_ladder(x: np.ndarray, dtype: str, keep_ratio, ladder):
    xd = to_device(x, dtype)
    sb, meta, ws = binding.alloc_buffers(xd, keep_ratio, len(ladder), binding.slicer_ladder_bit_set(ladder))
    ws.fill_(0xA5)
    sb.fill_(-1)
    meta.fill_(0xFF)
    binding.slicer_encode_ladder(xd, keep_ratio, ladder, sb, meta, ws)
    words = binding.slicer_stream_words(meta)
    return sb, meta, words


def gpu_decode(sb, meta, shape, dtype, n_blocks, use_header=True) -> np.ndarray:
    y = torch.full(shape, 7.0, dtype=torch.float32 if dtype == "f32" else torch.bfloat16, device="cuda")
    if use_header:
        binding.slicer_decode(sb, meta, y)
    else:
        binding.slicer_decode_as(sb, meta, y, n_blocks)
    torch.cuda.synchronize()
    return to_host(y)


def gpu_roundtrip(x: np.ndarray, dtype: str, keep_ratio, n_blocks, bit_set, budget, use_header=True):
    """(stream uint32[words], meta uint8[], y) from the HIP path."""
    sb, meta, words = gpu_encode(x, dtype, keep_ratio, n_blocks, bit_set, budget)
    y = torch.full(x.shape, 7.0, dtype=torch.float32 if dtype == "f32" else torch.bfloat16, device="cuda")
    if use_header:
        binding.slicer_decode(sb, meta, y)
    else:
        binding.slicer_decode_as(sb, meta, y, n_blocks)
    torch.cuda.synchronize()
    s = sb[:words].cpu().numpy().view(np.uint32)
    return s, meta.cpu().numpy(), to_host(y)
