"""The C-ABI library loads without a GPU and exports every symbol include/slicer.h
declares; host-only entry points (sizes, error strings, argument checks) behave."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2511_11608_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2511_11608_amd import build
        build.build()
    return binding.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "slicer.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(slicer_[a-z_]+)\s*\(", text)))


def test_exports_every_declared_symbol(lib):
    names = declared_symbols()
    assert {"slicer_sizes", "slicer_encode", "slicer_decode", "slicer_decode_as", "slicer_stream_words",
            "slicer_encode_path", "slicer_profile_events", "slicer_last_hip_error", "slicer_strerror",
            "slicer_encode_ladder", "slicer_ladder_bit_set", "slicer_bound", "slicer_check", "slicer_encode_ds",
            "slicer_sizes_pn", "slicer_encode_pn", "slicer_decode_as_pn", "slicer_check_pn", "slicer_encode_atkf"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n


def test_sizes_closed_form(lib):
    from paper_2511_11608_amd import binding, synth
    # workload 4: k = floor(0.1*4096) = 409, w = 12, q_bit = 8 -> ceil(409*20/32) = 256 words per row
    cap, mb, wb = binding.slicer_sizes(binding.SLICER_BF16, 16384, 4096, 0.10, 8, synth.BITS_2_TO_8)
    assert cap == 16384 * 256 * 4
    assert mb == 64 + 16 * 16384 + 18 * 16384 * 8
    assert wb >= cap
    # workload 2: k = 80281, w = 19
    cap, mb, _ = binding.slicer_sizes(binding.SLICER_F32, 32, 401408, 0.20, 16, synth.BITS_2_TO_8)
    assert cap == 32 * ((80281 * 27 + 31) // 32) * 4 and mb == 64 + 16 * 32 + 18 * 32 * 16


def test_argument_errors_and_strings(lib):
    from paper_2511_11608_amd import binding
    good = dict(dt=0, rows=2, row_len=8, keep_ratio=0.5, n_blocks=2, bit_set=0b111100)
    for kw, code in ((dict(dt=7), -2), (dict(rows=0), -1), (dict(row_len=0), -1), (dict(row_len=1 << 31), -1),
                     (dict(keep_ratio=-0.1), -1), (dict(keep_ratio=float("nan")), -1), (dict(n_blocks=0), -1),
                     (dict(n_blocks=65), -1), (dict(bit_set=0), -1), (dict(bit_set=1), -1), (dict(bit_set=1 << 17), -1)):
        a = dict(good); a.update(kw)
        with pytest.raises(binding.SlicerError) as ei:
            binding.slicer_sizes(a["dt"], a["rows"], a["row_len"], a["keep_ratio"], a["n_blocks"], a["bit_set"])
        assert ei.value.code == code
    assert lib.slicer_strerror(0) == b"ok"
    for code in (-1, -2, -3, -4, -5, -99):
        assert len(lib.slicer_strerror(code)) > 0
    # null pointers are rejected before anything is launched
    assert lib.slicer_encode(None, 0, 1, 8, 0.5, 1, 0b100, 1e-3, None, None, None, None) == -1
    assert lib.slicer_decode_as(None, None, None, 0, 1, 8, 1, None) == -1
    # the entry point without a workspace: shapes beyond its static scratch are refused before anything else
    assert lib.slicer_encode_static(None, 1, 16384, 4096, 0.1, 8, 0x1FC, 1e-3, None, None, None) == -5
    assert lib.slicer_encode_static(None, 1, 16, 4096, 0.1, 8, 0x1FC, 1e-3, None, None, None) == -1


def test_encode_path_by_shape(lib):
    from paper_2511_11608_amd import binding, synth
    B = synth.BITS_2_TO_8
    assert binding.slicer_encode_path(binding.SLICER_BF16, 16384, 4096, 0.10, 8, B) == 1     # LLM prefill
    assert binding.slicer_encode_path(binding.SLICER_BF16, 256, 8192, 0.10, 8, B) == 3       # AR decode step: one workgroup per row
    assert binding.slicer_encode_path(binding.SLICER_BF16, 16384, 8192, 0.10, 8, B) == 3     # the same rows in a large batch
    assert binding.slicer_encode_path(binding.SLICER_BF16, 300, 12288, 0.10, 8, B) == 3      # beyond one wavefront's row length
    assert binding.slicer_encode_path(binding.SLICER_F32, 12608, 768, 0.15, 8, B) == 1       # ViT tokens
    assert binding.slicer_encode_path(binding.SLICER_F32, 32, 401408, 0.20, 16, B) == 2      # ResNet stage 3
    assert binding.slicer_encode_path(binding.SLICER_F32, 1, 200704, 0.10, 4, B) == 2        # CNN map
    assert binding.slicer_encode_path(binding.SLICER_F32, 3, 4097, 0.5, 3, B) == 0           # odd length


def test_bound_matches_the_oracle_and_the_buffer_sizes(lib, oracle):
    """slicer_bound is host arithmetic: it must agree with the oracle's statement of Sec. 3.3 and
    with the worst-case buffer sizes, on the five workload shapes and a few odd ones."""
    from paper_2511_11608_amd import binding, synth
    B = synth.BITS_2_TO_8
    cases = [("f32", 1, 200704, 0.1, 4, B), ("f32", 32, 401408, 0.2, 16, B), ("f32", 12608, 768, 0.15, 8, B),
             ("bf16", 16384, 4096, 0.1, 8, B), ("bf16", 256, 8192, 0.1, 8, B), ("f32", 3, 1, 1.0, 1, 2),
             ("bf16", 7, 1000, 0.0, 64, 1 << 16), ("f32", 5, 4097, 0.37, 3, 0x1FFFE)]
    for dtype, R, N, keep, M, bits in cases:
        dt = binding.SLICER_F32 if dtype == "f32" else binding.SLICER_BF16
        got = binding.slicer_bound(dt, R, N, keep, M, bits)
        assert got == oracle.bound(dtype, R, N, keep, M, bits)
        cap, mb, _ = binding.slicer_sizes(dt, R, N, keep, M, bits)
        assert sum(got) == 8 * (cap + mb)
    with pytest.raises(binding.SlicerError):
        binding.slicer_bound(binding.SLICER_F32, 1, 16, 1.5, 2, B)


def test_ladder_bit_set(lib):
    from paper_2511_11608_amd import binding
    assert binding.slicer_ladder_bit_set([8, 6, 4, 2]) == (1 << 8) | (1 << 6) | (1 << 4) | (1 << 2)
    assert binding.slicer_ladder_bit_set([3, 3, 3]) == 1 << 3
    assert binding.slicer_ladder_bit_set([0, 3]) == 0 and binding.slicer_ladder_bit_set([17]) == 0


def test_sizes_pn(lib, oracle):
    from paper_2511_11608_amd import binding
    import ctypes as C
    for Mp, Mn in ((1, 1), (3, 8), (64, 1), (8, 8)):
        a, b, c = C.c_size_t(0), C.c_size_t(0), C.c_size_t(0)
        assert lib.slicer_sizes_pn(binding.SLICER_BF16, 100, 4096, 0.1, Mp, Mn, 0x1FC, C.byref(a), C.byref(b), C.byref(c)) == 0
        assert b.value == (64 + 16 * 100 + 9 * 100 * (Mp + Mn) + 7) // 8 * 8
        if Mp == Mn:
            assert (a.value, b.value, c.value) == binding.slicer_sizes(binding.SLICER_BF16, 100, 4096, 0.1, Mp, 0x1FC)
    a = C.c_size_t(0)
    assert lib.slicer_sizes_pn(binding.SLICER_BF16, 100, 4096, 0.1, 4, 0, 0x1FC, C.byref(a), None, None) == -1
    assert lib.slicer_sizes_pn(binding.SLICER_BF16, 100, 4096, 0.1, 4, 65, 0x1FC, C.byref(a), None, None) == -1
