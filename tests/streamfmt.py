"""Independent reader of the codec's wire format (version 1), in plain Python.

Written from the format description alone; it calls neither the oracle nor the HIP
library, so tests can use it to look inside a (stream, meta) pair produced by
either side: kept indices per block, integer codes, block sizes, bit counts.
"""
from __future__ import annotations

import numpy as np

MAGIC = 0x52434C53


def header(meta: np.ndarray) -> dict:
    m = np.ascontiguousarray(meta, np.uint8)
    u32 = lambda o: int(m[o:o + 4].view(np.uint32)[0])
    u64 = lambda o: int(m[o:o + 8].view(np.uint64)[0])
    return dict(magic=u32(0), version=u32(4), dtype=u32(8), M=u32(12), rows=u64(16), row_len=u64(24),
                k=u64(32), bit_set=u32(40), w=u32(44), total_words=u64(48), reserved=u64(56),
                M_neg=u32(56) or u32(12),          # 0 at offset 56: the negative class has M blocks too
                n_cols=u32(60))                    # non-zero: two-dimensional instance, blocks stored as CSR triples


def arrays(meta: np.ndarray) -> dict:
    h = header(meta)
    R, B = h["rows"], h["M"] + h["M_neg"]          # B blocks per row: positive class first
    m = np.ascontiguousarray(meta, np.uint8)
    o = 64
    row_off = m[o:o + 8 * R].view(np.uint64); o += 8 * R
    n_pos = m[o:o + 4 * R].view(np.uint32); o += 4 * R
    n_neg = m[o:o + 4 * R].view(np.uint32); o += 4 * R
    vmin = m[o:o + 4 * R * B].view(np.float32).reshape(R, B); o += 4 * R * B
    vmax = m[o:o + 4 * R * B].view(np.float32).reshape(R, B); o += 4 * R * B
    q = m[o:o + R * B].reshape(R, B); o += R * B
    size = (o + 7) // 8 * 8
    return dict(row_off=row_off, n_pos=n_pos, n_neg=n_neg, vmin=vmin, vmax=vmax, q=q, size=size)


def block_sizes(n_cls: int, M: int) -> list[int]:
    """Equal-cardinality sizes of one sign class: K, ..., K, K + remainder."""
    K = n_cls // M
    return [K] * (M - 1) + [n_cls - K * (M - 1)]


def _bits(words: np.ndarray, pos: int, n: int) -> int:
    v = 0
    for i in range(n):
        p = pos + i
        v |= ((int(words[p >> 5]) >> (p & 31)) & 1) << i
    return v


def parse_row(stream: np.ndarray, meta: np.ndarray, r: int) -> dict:
    """Blocks of row r: list (2M entries) of (indices, codes), plus bit accounting."""
    h = header(meta)
    a = arrays(meta)
    w = h["w"]
    sizes = block_sizes(int(a["n_pos"][r]), h["M"]) + block_sizes(int(a["n_neg"][r]), h["M_neg"])
    n = sum(sizes)
    words = np.ascontiguousarray(stream, np.uint32)[int(a["row_off"][r]):]
    ipos, cpos = 0, n * w
    blocks = []
    for b, cnt in enumerate(sizes):
        q = int(a["q"][r, b]) & 0x7F
        idx = [_bits(words, ipos + j * w, w) for j in range(cnt)]
        cod = [_bits(words, cpos + j * q, q) for j in range(cnt)]
        ipos += cnt * w
        cpos += cnt * q
        blocks.append((idx, cod))
    return dict(blocks=blocks, sizes=sizes, bits=cpos, words=(cpos + 31) // 32)


def parse_row_csr(stream: np.ndarray, meta: np.ndarray, r: int) -> dict:
    """Blocks of the two-dimensional instance r: list of (row pointers, columns, codes) per block."""
    h = header(meta)
    a = arrays(meta)
    wc, n_cols = h["w"], h["n_cols"]
    n_rows = h["row_len"] // n_cols
    wp = max(1, int(h["k"]).bit_length())                      # holds any value in 0..k
    sizes = block_sizes(int(a["n_pos"][r]), h["M"]) + block_sizes(int(a["n_neg"][r]), h["M_neg"])
    n = sum(sizes)
    words = np.ascontiguousarray(stream, np.uint32)[int(a["row_off"][r]):]
    ppos = 0
    ipos = len(sizes) * (n_rows + 1) * wp
    cpos = ipos + n * wc
    blocks = []
    for b, cnt in enumerate(sizes):
        q = int(a["q"][r, b]) & 0x7F
        ptr = [_bits(words, ppos + j * wp, wp) for j in range(n_rows + 1)]
        col = [_bits(words, ipos + j * wc, wc) for j in range(cnt)]
        cod = [_bits(words, cpos + j * q, q) for j in range(cnt)]
        ppos += (n_rows + 1) * wp
        ipos += cnt * wc
        cpos += cnt * q
        blocks.append((ptr, col, cod))
    return dict(blocks=blocks, sizes=sizes, bits=cpos, words=(cpos + 31) // 32)
