"""Randomised GPU parity: a few hundred seeded draws of shape, value structure, knobs and mode, each one
byte-exact against the oracle (stream, meta, decoded tensor).  The draws favour the widths and batch sizes at
which the library changes kernels or launch sequences (one wavefront or one workgroup per row, long-row stages,
one or two finishing launches) and value structures that stress the selection (post-ReLU zeros, outlier
channels, a handful of distinct values, per-row scales)."""
import numpy as np
import pytest

from paper_2511_11608_amd import synth
from tests.test_gpu_parity import B28, check, check_atkf, check_ds, check_ladder

pytestmark = pytest.mark.gpu

WIDTHS = {
    "f32": [256, 512, 768, 1024, 1280, 2048, 4096, 6144, 8192, 16384, 20000, 40960],
    "bf16": [256, 1024, 2048, 4096, 8192, 12288, 16384, 32768, 40960],
}


@pytest.mark.parametrize("seed", [101, 102, 103, 104])
def test_random_shapes_modes_and_values(oracle, seed):
    rng = np.random.default_rng(seed)
    for it in range(100):
        dtype = "f32" if rng.random() < 0.5 else "bf16"
        N = int(rng.choice(WIDTHS[dtype])) if rng.random() < 0.8 else int(rng.integers(1, 9000))
        rows = int(rng.choice([1, 2, 7, 33, 200, 256, 257, 300, 700])) if N <= 8192 else int(rng.choice([1, 2, 5, 33]))
        kind = int(rng.integers(0, 5))
        x = rng.standard_normal((rows, N)).astype(np.float32) * np.float32(10.0 ** rng.integers(-3, 4))
        if kind == 1:                                   # post-ReLU: one sign class, half zeros
            x = np.abs(x)
            x[rng.random((rows, N)) < 0.5] = 0
        elif kind == 2:                                 # outlier channels
            x[:, :: max(1, N // 8)] *= np.float32(40)
        elif kind == 3:                                 # a handful of distinct values: long runs of equal keys
            x = np.round(x * np.float32(4.0 / max(1e-30, float(np.abs(x).max())))) * np.float32(0.25)
        elif kind == 4:                                 # per-row scales
            x *= (10.0 ** rng.uniform(-2, 2, (rows, 1))).astype(np.float32)
        if dtype == "bf16":
            x = synth.f32_to_bf16_bits(x)
        keep = float(rng.choice([0.02, 0.05, 0.1, 0.15, 0.2, 0.3, 0.5, 1.0])) if rng.random() < 0.8 else float(rng.random())
        M = int(rng.choice([1, 2, 4, 8, 16, 32]))
        mode = int(rng.integers(0, 4))
        try:
            if mode == 0:
                check(oracle, x, dtype, keep, M, B28, float(10.0 ** rng.uniform(-5, -2)))
            elif mode == 1:
                check_ds(oracle, x, dtype, keep, M, B28, float(rng.choice([0.0, 0.2, 0.45, 5.0])))
            elif mode == 2:
                check_ladder(oracle, x, dtype, keep, [int(q) for q in rng.integers(1, 12, M)])
            else:
                check_atkf(oracle, x, dtype, keep, float(rng.random() * 0.9 + 0.05), M, int(rng.choice([1, 3, 8])), B28, 1e-3)
        except AssertionError as e:
            raise AssertionError(f"seed {seed} draw {it}: {dtype} [{rows} x {N}] kind {kind} keep {keep:.3f} M {M} mode {mode}: {e}")
