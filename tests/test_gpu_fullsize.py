"""GPU parity at the full sizes of the five workloads, in the launch configuration
bench.py times (same shapes, same knobs, same entry points).  The oracle is fast
enough (OpenMP over rows) to check every row: stream, meta and decoded tensor are
compared bit for bit.  The AR-decode workload is checked on a few of its 512 steps."""
import os

import numpy as np
import pytest

from paper_2511_11608_amd import synth
from tests.test_gpu_parity import check

pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_full_size_workload(oracle, cfg):
    wl = synth.make_config(cfg)
    check(oracle, wl.x, wl.dtype, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget, use_header=False)


@pytest.mark.parametrize("step", [0, 1, 255, 511])
def test_ar_decode_steps(oracle, step):
    wl = synth.ar_decode_step(seed=0, step=step)
    check(oracle, wl.x, wl.dtype, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget, use_header=True)


def test_size_accounting_llm_prefill(oracle):
    """Properties that hold at any size: offsets are the exclusive scan of the row word
    counts in closed form, and the payload stays under the paper's upper bound (Sec. 3.3)."""
    import torch
    from paper_2511_11608_amd import binding
    from tests import streamfmt
    from tests.gpu_util import gpu_encode
    wl = synth.llm_prefill(seed=5, rows=4096)
    sb, meta, words = gpu_encode(wl.x, wl.dtype, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget)
    m = meta.cpu().numpy()
    h, a = streamfmt.header(m), streamfmt.arrays(m)
    n = a["n_pos"].astype(np.int64) + a["n_neg"].astype(np.int64)
    assert np.all(n == h["k"])                       # no exact zeros in this workload: exact count (Sec. 3.1)
    M = wl.n_blocks
    q = (a["q"] & 0x7F).astype(np.int64)
    sizes = np.empty((wl.rows, 2 * M), np.int64)
    for s, cnt in ((0, a["n_pos"].astype(np.int64)), (1, a["n_neg"].astype(np.int64))):
        K = cnt // M
        sizes[:, s * M:(s + 1) * M] = K[:, None]
        sizes[:, s * M + M - 1] = cnt - K * (M - 1)
    bits = n * h["w"] + (sizes * q).sum(axis=1)
    row_words = (bits + 31) // 32
    assert np.array_equal(a["row_off"].astype(np.int64), np.cumsum(row_words) - row_words)
    assert int(row_words.sum()) == h["total_words"] == words
    assert np.all(bits <= n * (h["w"] + 8))
    assert np.all(a["vmin"] <= a["vmax"]) and np.all(a["vmin"][sizes > 0] > 0)
    for s in (0, M):        # blocks ordered by magnitude inside a class
        assert np.all(a["vmin"][:, s:s + M - 1] >= a["vmax"][:, s + 1:s + M])
