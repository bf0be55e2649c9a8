"""GPU parity at the full sizes of the five workloads, in the launch configuration
bench.py times (same shapes, same knobs, same entry points).  The oracle is fast
enough (OpenMP over rows) to check every row: stream, meta and decoded tensor are
compared bit for bit, on every one of the 512 steps of the AR-decode workload too."""
import os

import numpy as np
import pytest

from paper_2511_11608_amd import synth
from tests.test_gpu_parity import check, check_atkf

pytestmark = pytest.mark.gpu

THREADS = min(16, os.cpu_count() or 1)


@pytest.mark.parametrize("cfg", [1, 2, 3, 4])
def test_full_size_workload(oracle, cfg):
    wl = synth.make_config(cfg)
    check(oracle, wl.x, wl.dtype, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget, use_header=False)


@pytest.mark.parametrize("first", [0, 128, 256, 384])
def test_ar_decode_steps(oracle, first):
    """All 512 steps of the AR-decode workload (256 rows x 8192 bf16, a fresh seed per step), in four groups."""
    for step in range(first, first + 128):
        wl = synth.ar_decode_step(seed=0, step=step)
        check(oracle, wl.x, wl.dtype, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget, use_header=(step % 2 == 0))


@pytest.mark.parametrize("lam", [0.1, 0.7])
def test_full_size_llm_prefill_asymmetric(oracle, lam):
    """The headline tensor under the asymmetric thresholds of Sec. 3.1 (row-resident kernel with its
    second selection), every row against the oracle."""
    wl = synth.make_config(4)
    check_atkf(oracle, wl.x, wl.dtype, wl.keep_ratio, lam, wl.n_blocks, wl.n_blocks, wl.bit_set, wl.budget)


@pytest.mark.parametrize("lam", [0.1, 0.7])
def test_full_size_vit_tokens_asymmetric(oracle, lam):
    """The ViT tensor (fp32, the workload whose outlier channels make the asymmetry matter) under the
    asymmetric thresholds: row-resident kernel with the exact three-level selection, every row."""
    wl = synth.make_config(3)
    check_atkf(oracle, wl.x, wl.dtype, wl.keep_ratio, lam, wl.n_blocks, wl.n_blocks, wl.bit_set, wl.budget)


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


def test_tensor_beyond_4_gib(oracle):
    """Maximum sizes: a bf16 tensor of 4.9 GB (offsets of x, y and the slots cross 2^32 bytes), generated
    on the device.  Rows around the 4 GiB boundary, the first and the last are compared with the oracle
    run on those rows alone: meta slice, stream segment and decoded row, bit for bit."""
    import torch
    from paper_2511_11608_amd import binding
    from tests import streamfmt
    R, N, keep, M, bits, budget = 600_000, 4096, 0.1, 8, synth.BITS_2_TO_8, 1e-3
    g = torch.Generator(device="cuda").manual_seed(11)
    x = torch.empty((R, N), dtype=torch.bfloat16, device="cuda")
    for r0 in range(0, R, 50_000):                    # in pieces: the fp32 temporary stays small
        x[r0:r0 + 50_000] = (torch.randn((min(50_000, R - r0), N), generator=g, device="cuda") * 0.5).to(torch.bfloat16)
    sb, meta, ws = binding.alloc_buffers(x, keep, M, bits)
    binding.slicer_encode(x, keep, M, bits, budget, sb, meta, ws)
    words = binding.slicer_stream_words(meta)
    y = torch.full((R, N), 3.0, dtype=torch.bfloat16, device="cuda")
    binding.slicer_decode_as(sb, meta, y, M)
    torch.cuda.synchronize()
    m = meta.cpu().numpy()
    h, a = streamfmt.header(m), streamfmt.arrays(m)
    assert (h["rows"], h["row_len"], h["total_words"]) == (R, N, words)
    row_4gib = (1 << 32) // (2 * N)                   # first row whose bytes start at 4 GiB
    for r in (0, 1, row_4gib - 1, row_4gib, row_4gib + 1, R - 2, R - 1):
        xr = x[r:r + 1].view(torch.int16).cpu().numpy().view(np.uint16)
        s_ref, m_ref = oracle.encode(xr, "bf16", keep, M, bits, budget)
        a_ref = streamfmt.arrays(m_ref)
        for name in ("n_pos", "n_neg", "vmin", "vmax", "q"):
            assert np.array_equal(a_ref[name][0], a[name][r]), (r, name)
        off0 = int(a["row_off"][r])
        off1 = int(a["row_off"][r + 1]) if r + 1 < R else words
        seg = sb[off0:off1].cpu().numpy().view(np.uint32)
        assert np.array_equal(seg, s_ref), r
        y_ref = oracle.decode(s_ref, m_ref)
        assert np.array_equal(y[r:r + 1].view(torch.int16).cpu().numpy().view(np.uint16), y_ref), r
    # every row decoded: no element keeps the fill value
    assert not bool((y[::997] == 3.0).any())


@pytest.mark.parametrize("rows,N", [(2, 8_388_608), (1, 10_000_000)])
def test_very_long_rows(oracle, rows, N):
    """Row lengths at and beyond the limit of the long-row stages (1024 chunks of 8192 elements):
    the first shape runs them at their maximum, the second is served by the generic encoder."""
    rng = np.random.default_rng(N)
    x = rng.standard_normal((rows, N)).astype(np.float32)
    x[rng.random((rows, N)) < 0.3] = 0
    check(oracle, x, "f32", 0.05, 4, synth.BITS_2_TO_8, 1e-3, use_header=True)
