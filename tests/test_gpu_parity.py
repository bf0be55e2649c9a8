"""GPU parity: the HIP path, through the C ABI, against the CPU oracle.

Bit-exact on stream and meta (kept set, block membership, bitwidths, codes, ranges,
offsets) and on the decoded tensor, on seeded synthetic inputs shaped like the five
workloads (shrunk so the oracle finishes in seconds) plus the degenerate rows.
"""
import numpy as np
import pytest

from paper_2511_11608_amd import synth
from tests import streamfmt

pytestmark = pytest.mark.gpu

B28 = synth.BITS_2_TO_8


def explain_mismatch(s_ref, m_ref, s_gpu, m_gpu, rows):
    """First differing row and what differs there (for the assertion message)."""
    a, b = streamfmt.arrays(m_ref), streamfmt.arrays(m_gpu)
    for name in ("n_pos", "n_neg", "q", "vmin", "vmax", "row_off"):
        if not np.array_equal(a[name], b[name]):
            r = int(np.nonzero(np.atleast_1d((a[name] != b[name]).reshape(rows, -1).any(axis=1)))[0][0])
            return f"meta field {name} differs first at row {r}: ref {a[name][r]} gpu {b[name][r]}"
    if s_ref.size != s_gpu.size:
        return f"stream sizes differ: {s_ref.size} vs {s_gpu.size}"
    d = np.nonzero(s_ref != s_gpu)[0]
    if d.size:
        r = int(np.searchsorted(a["row_off"], d[0], side="right") - 1)
        pr, pg = streamfmt.parse_row(s_ref, m_ref, r), streamfmt.parse_row(s_gpu, m_gpu, r)
        for bi, (x, y) in enumerate(zip(pr["blocks"], pg["blocks"])):
            if x != y:
                return f"stream word {d[0]} (row {r}) differs; first differing block {bi}: ref {x} gpu {y}"
        return f"stream word {d[0]} (row {r}) differs"
    return "identical"


def check(oracle, wl_x, dtype, keep, M, bits, budget, use_header=True):
    from tests.gpu_util import gpu_encode, gpu_decode
    s_ref, m_ref = oracle.encode(wl_x, dtype, keep, M, bits, budget, n_threads=8)
    y_ref = oracle.decode(s_ref, m_ref, n_threads=8)
    sb, meta, words = gpu_encode(wl_x, dtype, keep, M, bits, budget)
    m_gpu = meta.cpu().numpy()
    # compare before decoding: the decoder is only ever fed a stream known to be well-formed
    assert np.array_equal(m_ref[:64], m_gpu[:64]), (streamfmt.header(m_ref), streamfmt.header(m_gpu))
    s_gpu = sb[:words].cpu().numpy().view(np.uint32)
    ok = np.array_equal(m_ref, m_gpu) and np.array_equal(s_ref, s_gpu)
    assert ok, explain_mismatch(s_ref, m_ref, s_gpu, m_gpu, wl_x.shape[0])
    y_gpu = gpu_decode(sb, meta, wl_x.shape, dtype, M, use_header)
    # decode: bit-identical (stronger than the 1e-6 relative bar)
    assert np.array_equal(y_ref.view(np.uint32 if dtype == "f32" else np.uint16),
                          y_gpu.view(np.uint32 if dtype == "f32" else np.uint16))


CASES = {
    "cnn_map": lambda: synth.cnn_map(seed=0),                                        # config 1, full size
    "cnn_map_ragged": lambda: synth.cnn_map(seed=1, rows=3, row_len=50_001),
    "resnet_2rows": lambda: synth.resnet_stage3(seed=0, rows=2),                      # config 2, real row length
    "vit": lambda: synth.vit_tokens(seed=0, rows=700),                               # config 3
    "llm": lambda: synth.llm_prefill(seed=0, rows=300),                              # config 4
    "ar_step": lambda: synth.ar_decode_step(seed=0, step=5, rows=64),                 # config 5
    "llm_wide": lambda: synth.llm_prefill(seed=2, rows=300, width=12288),            # between the row-resident and the long-row home ranges
    "vit_wide": lambda: synth.vit_tokens(seed=2, rows=200, width=8192),
    "vit_4096": lambda: synth.vit_tokens(seed=3, rows=200, width=4096),              # widest fp32 row of the row-resident kernel
    "llm_8192_batch": lambda: synth.llm_prefill(seed=4, rows=1500, width=8192),      # one workgroup per row in a batch that fills the chip
}


@pytest.mark.parametrize("name", list(CASES))
def test_workload_parity(oracle, name):
    wl = CASES[name]()
    check(oracle, wl.x, wl.dtype, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("N", [1, 2, 63, 64, 65, 257, 1000, 2048, 4096, 4097, 4104, 6144, 8192, 12288, 16384, 16385, 32768, 40000])
def test_adversarial_rows(oracle, dtype, N):
    x = synth.adversarial_rows(dtype, N, seed=N)
    for keep, M, bits, budget in ((0.0, 1, B28, 1e-3), (0.3, 2, B28, 1e-3), (1.0, 5, B28, 0.0),
                                  (0.11, 64, (1 << 1) | (1 << 16), 1e-6), (0.5, 3, 1 << 5, 1e-2)):
        check(oracle, x, dtype, keep, M, bits, budget, use_header=(M != 2))


@pytest.mark.parametrize("dtype,rows,N", [("bf16", 40, 4096), ("f32", 40, 768), ("f32", 3, 50_000), ("bf16", 2, 40_960),
                                          ("f32", 5, 4097), ("bf16", 3, 1001)])
@pytest.mark.parametrize("scale", [-105, -120, -143, 100])
def test_tiny_and_huge_magnitudes(oracle, dtype, rows, N, scale):
    """The quantiser works on each block's own scale (Sec. 3.2.1 defines the step for any non-zero range):
    tensors multiplied by 2^-105, 2^-120 or 2^-143 (block ranges far below what a scale L / range could hold
    in fp32; the second partly, the third wholly subnormal) and by 2^100 go through every encoder family
    bit-exactly."""
    rng = np.random.default_rng(N + scale)
    x = rng.standard_normal((rows, N)).astype(np.float32)
    x[rng.random((rows, N)) < 0.3] = 0
    x[:, :: 97] *= np.float32(40)
    x = np.ldexp(x, scale).astype(np.float32)
    if dtype == "bf16":
        x = synth.f32_to_bf16_bits(x)
    for keep, M, bits, budget in ((0.1, 8, B28, 1e-3), (0.3, 3, (1 << 2) | (1 << 12) | (1 << 16), 1e-7)):
        check(oracle, x, dtype, keep, M, bits, budget)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_random_parameters(oracle, dtype):
    rng = np.random.default_rng(123)
    for _ in range(12):
        rows = int(rng.integers(1, 9))
        N = int(rng.integers(1, 3000))
        x = rng.standard_normal((rows, N)).astype(np.float32) * np.float32(10.0 ** rng.integers(-3, 4))
        x[rng.random((rows, N)) < rng.random()] = 0
        if dtype == "bf16":
            x = synth.f32_to_bf16_bits(x)
        keep = float(rng.random())
        M = int(rng.integers(1, 20))
        bits = int(rng.integers(1, 1 << 16)) << 1
        budget = float(10.0 ** rng.uniform(-6, -1))
        check(oracle, x, dtype, keep, M, bits, budget)


def _mixed_rows(rng, rows, N, dtype):
    """Gaussian rows with per-row scale, plus sparse, constant, few-valued and one-sided rows."""
    x = rng.standard_normal((rows, N)).astype(np.float32) * (10.0 ** rng.uniform(-2, 2, (rows, 1))).astype(np.float32)
    x[1, rng.random(N) < 0.97] = 0                     # fewer non-zeros than k at most keep ratios
    x[2, :] = np.float32(1.5)                          # one key: every rank is a tie
    x[3, :] = rng.choice(np.array([-2.0, -1.0, 0.5, 1.0, 4.0], np.float32), N)
    x[4, :] = np.abs(x[4, :])                          # one sign class only
    x[5, :] = 0
    x[6, : N // 2] *= np.float32(1e-30)                # wide key range: coarse fine bins
    x[7, :] = rng.standard_normal(N).astype(np.float32) * np.float32(2e-30)   # block ranges just above 2^-100: huge scales
    return synth.f32_to_bf16_bits(x) if dtype == "bf16" else x


@pytest.mark.parametrize("dtype,N", [("bf16", 256), ("bf16", 4096), ("bf16", 8192), ("f32", 768), ("f32", 1280), ("f32", 2048),
                                     ("f32", 4096), ("f32", 8192), ("f32", 12288), ("bf16", 20480)])
def test_row_resident_variants(oracle, dtype, N):
    """Every variant of the one-wave-per-row and of the workgroup-per-row encoder (list in registers or
    LDS, short or long bitwidth ladders, up to 64 blocks, bf16 and fp32, 4 and 16 wavefronts per row) and
    both bit-field sources of the short-row decoder."""
    rng = np.random.default_rng(N)
    x = _mixed_rows(rng, 24, N, dtype)
    for keep, M, bits, budget in ((0.02, 1, B28, 1e-3), (0.1, 8, B28, 1e-3), (0.15, 32, B28, 5e-4),
                                  (0.25, 5, (1 << 1) | (1 << 16), 1e-5), (0.28, 3, 0xFE00, 1e-7),
                                  (0.45, 8, B28, 1e-3), (0.6, 2, 0x1FFFE, 1e-4), (1.0, 16, B28, 1e-2)):
        check(oracle, x, dtype, keep, M, bits, budget)


@pytest.mark.parametrize("dtype,N", [("bf16", 4096), ("f32", 768), ("f32", 4096), ("bf16", 8192), ("f32", 8192)])
def test_wide_dynamic_range_rows(oracle, dtype, N):
    """Magnitudes spread evenly over many octaves: the row kernel's histogram window covers 16
    octaves below the row's largest value, so these rows put rank k-1 inside the window, on its
    last bin, and below it (second, coarser pass), with and without zeros under it."""
    x = _wide_range_rows(N, dtype)
    for keep, M in ((0.05, 4), (0.3, 8), (0.5, 3), (0.9, 8), (1.0, 2)):
        check(oracle, x, dtype, keep, M, B28, 1e-3)


def _wide_range_rows(N, dtype):
    rng = np.random.default_rng(7 * N)
    rows = 12
    spans = np.array([4, 12, 15.9, 16.0, 16.1, 17, 24, 40, 60, 90, 120, 30], np.float32)[:, None]
    mag = np.exp2(-spans * rng.random((rows, N)).astype(np.float32)) * np.float32(8.0)
    x = (mag * rng.choice(np.array([-1.0, 1.0], np.float32), (rows, N))).astype(np.float32)
    x[11, rng.random(N) < 0.5] = 0                      # zeros below a wide range
    x[10, 0] = np.float32(3e38)                         # one huge value on top of 120 octaves
    return synth.f32_to_bf16_bits(x) if dtype == "bf16" else x


def check_ladder(oracle, x, dtype, keep, ladder):
    from tests.gpu_util import gpu_encode_ladder, gpu_decode
    s_ref, m_ref = oracle.encode_ladder(x, dtype, keep, ladder, n_threads=8)
    y_ref = oracle.decode(s_ref, m_ref, n_threads=8)
    sb, meta, words = gpu_encode_ladder(x, dtype, keep, ladder)
    m_gpu = meta.cpu().numpy()
    assert np.array_equal(m_ref[:64], m_gpu[:64]), (streamfmt.header(m_ref), streamfmt.header(m_gpu))
    s_gpu = sb[:words].cpu().numpy().view(np.uint32)
    ok = np.array_equal(m_ref, m_gpu) and np.array_equal(s_ref, s_gpu)
    assert ok, explain_mismatch(s_ref, m_ref, s_gpu, m_gpu, x.shape[0])
    y_gpu = gpu_decode(sb, meta, x.shape, dtype, len(ladder))
    assert np.array_equal(y_ref.view(np.uint32 if dtype == "f32" else np.uint16),
                          y_gpu.view(np.uint32 if dtype == "f32" else np.uint16))


@pytest.mark.parametrize("name", ["cnn_map_ragged", "resnet_2rows", "vit", "llm", "ar_step"])
def test_ladder_mode_workloads(oracle, name):
    """Fixed multi-level mode (Sec. 4.1) on every kernel family: row-resident, long-row stages, generic."""
    wl = CASES[name]()
    for ladder in ([8, 6, 5, 4, 3, 3, 2, 2], [4], [16, 1], [2, 9, 2, 9, 5]):
        check_ladder(oracle, wl.x, wl.dtype, wl.keep_ratio, ladder)


@pytest.mark.parametrize("dtype,N", [("bf16", 4096), ("f32", 768), ("bf16", 1000), ("f32", 40000)])
def test_ladder_mode_mixed_rows(oracle, dtype, N):
    rng = np.random.default_rng(N + 1)
    x = _mixed_rows(rng, 12, N, dtype)
    for keep, ladder in ((0.1, [8, 7, 6, 5, 4, 3, 2, 2]), (1.0, [3, 2]), (0.3, list(range(16, 0, -1)) * 2), (0.0, [5])):
        check_ladder(oracle, x, dtype, keep, ladder)


def check_ds(oracle, x, dtype, keep, M, bits, delta):
    from tests.gpu_util import gpu_encode_ds, gpu_decode
    s_ref, m_ref = oracle.encode_ds(x, dtype, keep, M, bits, delta, n_threads=8)
    y_ref = oracle.decode(s_ref, m_ref, n_threads=8)
    sb, meta, words = gpu_encode_ds(x, dtype, keep, M, bits, delta)
    m_gpu = meta.cpu().numpy()
    assert np.array_equal(m_ref[:64], m_gpu[:64]), (streamfmt.header(m_ref), streamfmt.header(m_gpu))
    s_gpu = sb[:words].cpu().numpy().view(np.uint32)
    ok = np.array_equal(m_ref, m_gpu) and np.array_equal(s_ref, s_gpu)
    assert ok, explain_mismatch(s_ref, m_ref, s_gpu, m_gpu, x.shape[0])
    y_gpu = gpu_decode(sb, meta, x.shape, dtype, M)
    assert np.array_equal(y_ref.view(np.uint32 if dtype == "f32" else np.uint16),
                          y_gpu.view(np.uint32 if dtype == "f32" else np.uint16))


@pytest.mark.parametrize("name", ["cnn_map_ragged", "resnet_2rows", "vit", "llm", "ar_step"])
def test_ds_guard_workloads(oracle, name):
    """The paper's DS guard (Eq. "DS", greedy descent) on every kernel family."""
    wl = CASES[name]()
    for delta in (0.0, 0.26, 0.45, 1e6):
        check_ds(oracle, wl.x, wl.dtype, wl.keep_ratio, wl.n_blocks, wl.bit_set, delta)


@pytest.mark.parametrize("dtype,N", [("bf16", 4096), ("f32", 768), ("bf16", 1000), ("f32", 40000),
                                     ("bf16", 8192), ("f32", 8192), ("bf16", 20480)])    # the last three: one workgroup per row
def test_ds_guard_mixed_rows(oracle, dtype, N):
    rng = np.random.default_rng(N + 2)
    x = _mixed_rows(rng, 12, N, dtype)
    for keep, M, bits, delta in ((0.1, 8, B28, 0.3), (1.0, 3, 0x1FFFE, 0.4), (0.3, 32, (1 << 1) | (1 << 9) | (1 << 16), 0.5),
                                 (0.2, 2, 1 << 6, 0.0), (0.0, 1, B28, 0.1)):
        check_ds(oracle, x, dtype, keep, M, bits, delta)


@pytest.mark.parametrize("name", ["cnn_map_ragged", "resnet_2rows", "vit", "llm", "ar_step"])
def test_separate_block_counts_workloads(oracle, name):
    """M(+) != M(-) (Sec. 3.3) on every kernel family, through both decode entry points and the checker."""
    import torch
    from paper_2511_11608_amd import binding
    from paper_2511_11608_amd.devmem import to_device, to_host
    wl = CASES[name]()
    xd = to_device(wl.x, wl.dtype)
    for Mp, Mn in ((1, 5), (7, 2), (16, 3), (4, 4)):
        s_ref, m_ref = oracle.encode_pn(wl.x, wl.dtype, wl.keep_ratio, Mp, Mn, wl.bit_set, wl.budget, n_threads=8)
        y_ref = oracle.decode(s_ref, m_ref, n_threads=8)
        sb, meta, ws = binding.alloc_buffers_pn(xd, wl.keep_ratio, Mp, Mn, wl.bit_set)
        ws.fill_(0xA5); sb.fill_(-1); meta.fill_(0xFF)
        binding.slicer_encode_pn(xd, wl.keep_ratio, Mp, Mn, wl.bit_set, wl.budget, sb, meta, ws)
        words = binding.slicer_stream_words(meta)
        m_gpu = meta.cpu().numpy()
        s_gpu = sb[:words].cpu().numpy().view(np.uint32)
        assert np.array_equal(m_ref[:64], m_gpu[:64]), (streamfmt.header(m_ref), streamfmt.header(m_gpu))
        ok = np.array_equal(m_ref, m_gpu) and np.array_equal(s_ref, s_gpu)
        assert ok, explain_mismatch(s_ref, m_ref, s_gpu, m_gpu, wl.x.shape[0])
        binding.slicer_check_pn(meta, words, xd, Mp, Mn)
        for via_header in (True, False):
            y = torch.full_like(xd, 7.0)
            if via_header:
                binding.slicer_decode(sb, meta, y)
            else:
                binding.slicer_decode_as_pn(sb, meta, y, Mp, Mn)
            torch.cuda.synchronize()
            yv = np.uint32 if wl.dtype == "f32" else np.uint16
            assert np.array_equal(y_ref.view(yv), to_host(y).view(yv))


@pytest.mark.parametrize("dtype,N", [("bf16", 4096), ("f32", 768), ("bf16", 1000), ("f32", 40000)])
def test_separate_block_counts_mixed_rows(oracle, dtype, N):
    from paper_2511_11608_amd import binding
    from paper_2511_11608_amd.devmem import to_device
    rng = np.random.default_rng(N + 3)
    x = _mixed_rows(rng, 12, N, dtype)
    xd = to_device(x, dtype)
    for keep, Mp, Mn, bits in ((0.1, 8, 3, B28), (1.0, 1, 9, 0x1FFFE), (0.3, 40, 24, B28), (0.02, 2, 1, 1 << 4)):
        s_ref, m_ref = oracle.encode_pn(x, dtype, keep, Mp, Mn, bits, 1e-3, n_threads=8)
        sb, meta, ws = binding.alloc_buffers_pn(xd, keep, Mp, Mn, bits)
        ws.fill_(0x5A); sb.fill_(-1); meta.fill_(0xFF)
        binding.slicer_encode_pn(xd, keep, Mp, Mn, bits, 1e-3, sb, meta, ws)
        words = binding.slicer_stream_words(meta)
        m_gpu = meta.cpu().numpy()
        s_gpu = sb[:words].cpu().numpy().view(np.uint32)
        ok = np.array_equal(m_ref, m_gpu) and np.array_equal(s_ref, s_gpu)
        assert ok, explain_mismatch(s_ref, m_ref, s_gpu, m_gpu, x.shape[0])


def check_atkf(oracle, x, dtype, keep, lam, Mp, Mn, bits, budget):
    import torch
    from paper_2511_11608_amd import binding
    from paper_2511_11608_amd.devmem import to_device, to_host
    xd = to_device(x, dtype)
    s_ref, m_ref = oracle.encode_atkf(x, dtype, keep, lam, Mp, Mn, bits, budget, n_threads=8)
    y_ref = oracle.decode(s_ref, m_ref, n_threads=8)
    sb, meta, ws = binding.alloc_buffers_pn(xd, keep, Mp, Mn, bits)
    ws.fill_(0x3C); sb.fill_(-1); meta.fill_(0xFF)
    binding.slicer_encode_atkf(xd, keep, lam, Mp, Mn, bits, budget, sb, meta, ws)
    words = binding.slicer_stream_words(meta)
    m_gpu = meta.cpu().numpy()
    s_gpu = sb[:words].cpu().numpy().view(np.uint32)
    assert np.array_equal(m_ref[:64], m_gpu[:64]), (streamfmt.header(m_ref), streamfmt.header(m_gpu))
    ok = np.array_equal(m_ref, m_gpu) and np.array_equal(s_ref, s_gpu)
    assert ok, explain_mismatch(s_ref, m_ref, s_gpu, m_gpu, x.shape[0])
    y = torch.full_like(xd, 7.0)
    binding.slicer_decode(sb, meta, y)
    torch.cuda.synchronize()
    yv = np.uint32 if dtype == "f32" else np.uint16
    assert np.array_equal(y_ref.view(yv), to_host(y).view(yv))


@pytest.mark.parametrize("name", ["cnn_map_ragged", "resnet_2rows", "vit", "llm", "ar_step"])
def test_asymmetric_thresholds_workloads(oracle, name):
    """Sec. 3.1 with lambda > 0 (second selection over a subset of the row), and lambda = 0 through
    the same entry point (the fast kernels)."""
    wl = CASES[name]()
    x = wl.x[:24] if wl.x.shape[0] > 24 else wl.x
    for lam in (0.0, 0.05, 0.5, 0.95):
        check_atkf(oracle, x, wl.dtype, wl.keep_ratio, lam, wl.n_blocks, wl.n_blocks, wl.bit_set, wl.budget)


@pytest.mark.parametrize("dtype,N", [("bf16", 4096), ("f32", 768), ("bf16", 1000), ("f32", 5000), ("f32", 2048), ("f32", 4096), ("f32", 64)])
def test_asymmetric_thresholds_mixed_rows(oracle, dtype, N):
    """Degenerate rows (sparse, constant, few-valued, one-sided, all zero) and a mostly negative row, where
    the strict set is larger than k and is cut back."""
    rng = np.random.default_rng(N + 4)
    x = _mixed_rows(rng, 12, N, dtype)
    neg_row = (rng.standard_normal(N) - 0.8).astype(np.float32)
    x[8] = synth.f32_to_bf16_bits(neg_row) if dtype == "bf16" else neg_row
    for keep, lam, Mp, Mn in ((0.1, 0.3, 8, 8), (0.02, 0.9, 1, 3), (0.5, 0.1, 5, 2), (1.0, 0.5, 4, 4), (0.0, 0.2, 2, 2)):
        check_atkf(oracle, x, dtype, keep, lam, Mp, Mn, B28, 1e-3)


@pytest.mark.parametrize("dtype,N", [("bf16", 4096), ("bf16", 8192), ("f32", 768), ("f32", 4096)])
def test_asymmetric_thresholds_wide_range(oracle, dtype, N):
    """Rows whose tau or last fill key lies more than 16 octaves below the largest value: bf16 rows are then
    redone by the generic kernel under the same rule (the row-resident kernel takes both selections from a
    window of single keys), fp32 rows take the wider first level of the exact selection; next to rows that
    stay on the ordinary path."""
    x = _wide_range_rows(N, dtype)
    for keep, lam, M in ((0.05, 0.2, 4), (0.3, 0.6, 8), (0.9, 0.95, 8), (1.0, 0.5, 2)):
        check_atkf(oracle, x, dtype, keep, lam, M, M, B28, 1e-3)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_asymmetric_thresholds_random_parameters(oracle, dtype):
    """Random row lengths, keep ratios, asymmetry factors, block counts and value scales; few-valued rows
    make long runs of equal keys at both selections (the cut of the ties in index order)."""
    rng = np.random.default_rng(321)
    for it in range(16):
        rows = int(rng.integers(1, 9))
        N = int(rng.integers(1, 400)) * 8 if it % 2 == 0 else int(rng.integers(1, 3000))
        x = rng.standard_normal((rows, N)).astype(np.float32) * np.float32(10.0 ** rng.integers(-3, 4))
        if it % 3 == 0:
            x = np.round(x * np.float32(2.0 / max(1e-30, float(np.abs(x).max())))) * np.float32(0.5)     # a handful of distinct values
        x[rng.random((rows, N)) < rng.random() * 0.8] = 0
        if dtype == "bf16":
            x = synth.f32_to_bf16_bits(x)
        keep = float(rng.random())
        lam = float(rng.random() * 0.98 + 0.01)
        Mp, Mn = int(rng.integers(1, 12)), int(rng.integers(1, 12))
        check_atkf(oracle, x, dtype, keep, lam, Mp, Mn, B28, float(10.0 ** rng.uniform(-5, -2)))


def test_concurrent_calls_on_three_streams(oracle):
    """Independent batches encoded and decoded on three streams at once (each call with buffers of its
    own, as the benchmark does): every result is the oracle's, whatever the overlap."""
    import torch
    from paper_2511_11608_amd import binding
    from paper_2511_11608_amd.devmem import to_device, to_host
    wls = [synth.llm_prefill(seed=11 + i, rows=700) for i in range(3)] + [synth.vit_tokens(seed=21 + i, rows=500) for i in range(3)]
    refs = []
    for wl in wls:
        s_ref, m_ref = oracle.encode(wl.x, wl.dtype, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget, n_threads=8)
        refs.append((s_ref, m_ref, oracle.decode(s_ref, m_ref, n_threads=8)))
    xs = [to_device(wl.x, wl.dtype) for wl in wls]
    bufs = [binding.alloc_buffers(x, wl.keep_ratio, wl.n_blocks, wl.bit_set) for x, wl in zip(xs, wls)]
    ys = [torch.empty_like(x) for x in xs]
    streams = [torch.cuda.Stream() for _ in range(3)]
    torch.cuda.synchronize()
    for rep in range(4):
        for b, y in zip(bufs, ys):
            b[0].fill_(-1); b[1].fill_(0xFF); y.fill_(3.0)
        torch.cuda.synchronize()
        for i, (wl, x, (sb, meta, ws), y) in enumerate(zip(wls, xs, bufs, ys)):
            st = streams[i % 3]
            binding.slicer_encode(x, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget, sb, meta, ws, stream=st)
            binding.slicer_decode_as(sb, meta, y, wl.n_blocks, stream=st)
        torch.cuda.synchronize()
        for wl, (sb, meta, ws), y, (s_ref, m_ref, y_ref) in zip(wls, bufs, ys, refs):
            assert np.array_equal(meta.cpu().numpy(), m_ref)
            assert np.array_equal(sb[:s_ref.size].cpu().numpy().view(np.uint32), s_ref)
            yv = np.uint32 if wl.dtype == "f32" else np.uint16
            assert np.array_equal(to_host(y).view(yv), y_ref.view(yv))


def test_encode_is_deterministic():
    from tests.gpu_util import gpu_roundtrip
    wl = synth.llm_prefill(seed=3, rows=64)
    a = gpu_roundtrip(wl.x, wl.dtype, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget)
    b = gpu_roundtrip(wl.x, wl.dtype, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget)
    assert all(np.array_equal(u, v) for u, v in zip(a, b))


def test_error_codes():
    import torch
    from paper_2511_11608_amd import binding
    x = torch.zeros(4, 16, device="cuda")
    sb, meta, ws = binding.alloc_buffers(x, 0.5, 2, B28)
    for kw in (dict(keep_ratio=1.5), dict(n_blocks=0), dict(n_blocks=65), dict(bit_set=1), dict(budget=-1.0)):
        args = dict(keep_ratio=0.5, n_blocks=2, bit_set=B28, budget=1e-3); args.update(kw)
        with pytest.raises(binding.SlicerError):
            binding.slicer_encode(x, args["keep_ratio"], args["n_blocks"], args["bit_set"], args["budget"], sb, meta, ws)
    meta.zero_()
    with pytest.raises(binding.SlicerError) as ei:
        binding.slicer_decode(sb, meta, x)
    assert ei.value.code == -4


def test_check_accepts_encoder_output_and_rejects_forged_meta(oracle):
    """slicer_check on what the encoder wrote (GPU and oracle bytes alike) and on single-field
    forgeries of it.  Forged buffers only go to the checker, never to a decode call."""
    import torch
    from paper_2511_11608_amd import binding
    from tests.gpu_util import gpu_encode
    wl = synth.llm_prefill(seed=7, rows=40)
    sb, meta, words = gpu_encode(wl.x, wl.dtype, wl.keep_ratio, wl.n_blocks, wl.bit_set, wl.budget)
    y = torch.empty(wl.x.shape, dtype=torch.bfloat16, device="cuda")
    M, R = wl.n_blocks, wl.rows
    binding.slicer_check(meta, words, y, M)
    s_ref, m_ref = oracle.encode(wl.x, wl.dtype, wl.keep_ratio, M, wl.bit_set, wl.budget)
    binding.slicer_check(torch.from_numpy(m_ref).cuda(), int(s_ref.size), y, M)

    good = meta.cpu().numpy().copy()
    a = streamfmt.arrays(good)
    o_npos, o_q = 64 + 8 * R, 64 + 16 * R + 16 * R * M

    def forged(edit):
        m = good.copy()
        edit(m)
        return torch.from_numpy(m).cuda()

    def expect_reject(m, w=words, shape_like=y, blocks=M):
        with pytest.raises(binding.SlicerError) as ei:
            binding.slicer_check(m, w, shape_like, blocks)
        assert ei.value.code == -4

    expect_reject(meta, words - 1)                                                  # fewer words than the header claims
    expect_reject(forged(lambda m: m.__setitem__(0, m[0] ^ 1)))                     # magic
    expect_reject(forged(lambda m: m[48:56].view(np.uint64).__setitem__(0, words + 5)))   # total_words
    expect_reject(forged(lambda m: m[64 + 8 * 3: 64 + 8 * 4].view(np.uint64).__setitem__(0, 1 << 40)))   # a row offset
    expect_reject(forged(lambda m: m[o_npos + 4 * 5: o_npos + 4 * 6].view(np.uint32).__setitem__(0, 4000)))   # n_pos > k
    expect_reject(forged(lambda m: m[o_npos + 4 * 5: o_npos + 4 * 6].view(np.uint32).__setitem__(0, int(a["n_pos"][5]) + 1)))
    expect_reject(forged(lambda m: m.__setitem__(o_q + 7, 0)))                      # bitwidth 0
    expect_reject(forged(lambda m: m.__setitem__(o_q + 7, 9)))                      # bitwidth outside the header's set
    expect_reject(forged(lambda m: m.__setitem__(o_q + 7, int(good[o_q + 7]) ^ 1 if (int(good[o_q + 7]) ^ 1) in range(2, 9) else 8 if good[o_q + 7] != 8 else 7)))
    expect_reject(meta, words, torch.empty((R, 2048), dtype=torch.bfloat16, device="cuda"))          # other row length
    expect_reject(meta, words, y, M + 1)


@pytest.mark.parametrize("dtype,N,rows", [("bf16", 4096, 700), ("f32", 768, 900), ("bf16", 8192, 96), ("bf16", 8192, 2000)])
def test_one_workspace_reused_across_calls(oracle, dtype, N, rows):
    """The workspace keeps threshold hints from one call to the next (and nothing else that matters): the
    same buffers serve tensors of very different scale, sparsity and knobs in turn, so every call starts
    from the previous call's hints, good, stale or far off.  Every call is compared with the oracle."""
    import torch
    from paper_2511_11608_amd import binding
    from paper_2511_11608_amd.devmem import to_device
    rng = np.random.default_rng(N + rows)
    base = rng.standard_normal((rows, N)).astype(np.float32)
    variants = [base, base * np.float32(300), base * np.float32(1e-3), np.where(rng.random((rows, N)) < 0.93, 0, base).astype(np.float32),
                base, np.abs(base) * (10.0 ** rng.uniform(-3, 3, (rows, 1))).astype(np.float32), base * np.float32(300)]
    keep_max, M, bits = 0.2, 8, B28
    x0 = to_device(synth.f32_to_bf16_bits(base) if dtype == "bf16" else base, dtype)
    sb, meta, ws = binding.alloc_buffers(x0, keep_max, M, bits)      # sized for the largest keep ratio used
    ws.fill_(0x5A)
    for i, xf in enumerate(variants):
        x = synth.f32_to_bf16_bits(xf) if dtype == "bf16" else xf
        keep = (0.1, 0.2, 0.05)[i % 3]
        s_ref, m_ref = oracle.encode(x, dtype, keep, M, bits, 1e-3, n_threads=8)
        sb.fill_(-1); meta.fill_(0xFF)
        xd = to_device(x, dtype)
        binding.slicer_encode(xd, keep, M, bits, 1e-3, sb, meta, ws)
        words = binding.slicer_stream_words(meta)
        mb = m_ref.size
        m_gpu = meta[:mb].cpu().numpy()
        s_gpu = sb[:words].cpu().numpy().view(np.uint32)
        ok = np.array_equal(m_ref, m_gpu) and np.array_equal(s_ref, s_gpu)
        assert ok, (i, explain_mismatch(s_ref, m_ref, s_gpu, m_gpu, rows))


def check_csr(oracle, x, dtype, n_rows, n_cols, keep, M, bits, budget):
    import torch
    from paper_2511_11608_amd import binding
    from paper_2511_11608_amd.devmem import to_device, to_host
    xd = to_device(x, dtype)
    s_ref, m_ref = oracle.encode_csr(x, dtype, n_rows, n_cols, keep, M, bits, budget, n_threads=8)
    y_ref = oracle.decode(s_ref, m_ref, n_threads=8)
    sb, meta, ws = binding.alloc_buffers_csr(xd, n_rows, n_cols, keep, M, bits)
    ws.fill_(0x7E); sb.fill_(-1); meta.fill_(0xFF)
    binding.slicer_encode_csr(xd, n_rows, n_cols, keep, M, bits, budget, sb, meta, ws)
    words = binding.slicer_stream_words(meta)
    m_gpu = meta.cpu().numpy()
    s_gpu = sb[:words].cpu().numpy().view(np.uint32)
    assert np.array_equal(m_ref[:64], m_gpu[:64]), (streamfmt.header(m_ref), streamfmt.header(m_gpu))
    assert np.array_equal(m_ref, m_gpu) and np.array_equal(s_ref, s_gpu)
    # the checker takes what the encoder wrote, and neither a flat-format claim nor a short buffer
    binding.slicer_check_csr(meta, words, xd, n_rows, n_cols, M)
    if words:
        with pytest.raises(binding.SlicerError):
            binding.slicer_check_csr(meta, words - 1, xd, n_rows, n_cols, M)
    with pytest.raises(binding.SlicerError):
        binding.slicer_check(meta, words, xd, M)
    yv = np.uint32 if dtype == "f32" else np.uint16
    for via_header in (True, False):
        y = torch.full_like(xd, 7.0)
        if via_header:
            binding.slicer_decode(sb, meta, y)
        else:
            binding.slicer_decode_as_csr(sb, meta, y, n_rows, n_cols, M)
        torch.cuda.synchronize()
        assert np.array_equal(y_ref.view(yv), to_host(y).view(yv))


@pytest.mark.parametrize("dtype,inst,n_rows,n_cols", [("f32", 1, 64, 3136), ("f32", 3, 197, 768), ("bf16", 2, 128, 4096),
                                                      ("f32", 2, 5, 7), ("bf16", 4, 1, 1000), ("f32", 2, 1000, 1),
                                                      ("bf16", 1, 3, 20000), ("f32", 1, 2048, 100),
                                                      ("f32", 4, 4096, 50), ("bf16", 40, 300, 33)])   # many short tensor rows: 16 and 11 per decode workgroup
def test_two_dimensional_instances_csr(oracle, dtype, inst, n_rows, n_cols):
    """Sec. 3.2 step 3: whole n_rows x n_cols tensors as one instance, blocks stored as CSR(values, columns,
    row pointers); the first shape is the CNN map of workload 1 as 64 channels x 56*56, the second a ViT
    image (197 tokens x 768), the third an LLM slab (128 tokens x 4096).  Stream, meta and the decoded
    tensor bit for bit against the oracle, through both decode entry points."""
    T = n_rows * n_cols
    rng = np.random.default_rng(T + inst)
    x = rng.standard_normal((inst, T)).astype(np.float32)
    x[rng.random((inst, T)) < 0.45] = 0
    x[:, :: 211] *= np.float32(25)
    x[-1, : T // 3] = 0                                   # empty tensor rows
    if dtype == "bf16":
        x = synth.f32_to_bf16_bits(x)
    for keep, M, bits, budget in ((0.1, 4, B28, 1e-3), (0.5, 8, B28, 5e-4), (1.0, 3, (1 << 3) | (1 << 16), 1e-6), (0.0, 2, B28, 1e-3)):
        check_csr(oracle, x, dtype, n_rows, n_cols, keep, M, bits, budget)
