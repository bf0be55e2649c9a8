"""Seeded synthetic intermediate features (IFs) shaped like the paper's workloads.

Input generation only: nothing here belongs to the codec's arithmetic.  Both the
HIP path and the CPU oracle are fed from this module so that they see the same
bytes.  bf16 tensors are carried as ``uint16`` bit patterns (numpy has no bf16).

The five workloads stand in for the CNN / ViT / LLM features the paper measures
on (Sec. 4.1 lists the real models and datasets; neither is available here):

1. one post-ReLU CNN map, fp32 [1,64,56,56]: half exact zeros, rest |N(0,1)|;
2. ResNet-50 stage-3 style batch, fp32 [32,512,28,28]: 60 % zeros, rest
   half-normal with a per-channel sigma ~ U(0.2, 2); one codec row per sample;
3. ViT-B/16 style tokens, fp32 [64,197,768]: signed N(0,1), two fixed outlier
   channels x30; one codec row per token;
4. LLM prefill hidden states, bf16 [8,2048,4096]: 90 % N(0, sigma=0.5), 10 %
   Laplace(0, b=0.5), 0.1 % of the channels are outliers x50; row per token;
5. AR decode step, bf16 [256, 8192]: same distribution as 4, fresh seed per step.
"""
from __future__ import annotations

from dataclasses import dataclass
import numpy as np

BITS_2_TO_8 = sum(1 << q for q in range(2, 9))


@dataclass
class Workload:
    name: str
    x: np.ndarray          # float32 [rows,row_len] or uint16 (bf16 bits) [rows,row_len]
    dtype: str             # "f32" | "bf16"
    rows: int
    row_len: int
    keep_ratio: float
    n_blocks: int
    bit_set: int
    budget: float

    @property
    def nbytes(self) -> int:
        return self.x.nbytes

    def as_float32(self) -> np.ndarray:
        """Exact fp32 view of the values (bf16 widens exactly)."""
        if self.dtype == "f32":
            return self.x
        return (self.x.astype(np.uint32) << 16).view(np.float32)


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even narrowing of finite fp32 to bf16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> 16) & 1
    return ((u + 0x7FFF + lsb) >> 16).astype(np.uint16)


def bf16_bits_to_f32(h: np.ndarray) -> np.ndarray:
    return (h.astype(np.uint32) << 16).view(np.float32)


def _llm_rows(rng: np.random.Generator, rows: int, width: int) -> np.ndarray:
    g = rng.standard_normal((rows, width), dtype=np.float32) * np.float32(0.5)
    lap = rng.laplace(0.0, 0.5, size=(rows, width)).astype(np.float32)
    pick = rng.random((rows, width), dtype=np.float32) < np.float32(0.1)
    x = np.where(pick, lap, g)
    n_out = max(1, int(round(0.001 * width)))
    chans = rng.choice(width, size=n_out, replace=False)
    x[:, chans] *= np.float32(50.0)
    return f32_to_bf16_bits(x)


def cnn_map(seed: int = 0, rows: int = 1, row_len: int = 64 * 56 * 56) -> Workload:
    rng = np.random.default_rng(seed)
    g = np.abs(rng.standard_normal((rows, row_len), dtype=np.float32))
    mask = rng.random((rows, row_len), dtype=np.float32) < np.float32(0.5)
    x = np.where(mask, g, np.float32(0.0)).astype(np.float32)
    return Workload("cnn_map_f32", x, "f32", rows, row_len, 0.10, 4, BITS_2_TO_8, 1e-3)


def resnet_stage3(seed: int = 0, rows: int = 32, channels: int = 512, hw: int = 28 * 28) -> Workload:
    rng = np.random.default_rng(seed)
    sigma = rng.uniform(0.2, 2.0, size=channels).astype(np.float32)
    g = np.abs(rng.standard_normal((rows, channels, hw), dtype=np.float32)) * sigma[None, :, None]
    mask = rng.random((rows, channels, hw), dtype=np.float32) < np.float32(0.4)
    x = np.where(mask, g, np.float32(0.0)).astype(np.float32).reshape(rows, channels * hw)
    return Workload("resnet_stage3_f32", x, "f32", rows, channels * hw, 0.20, 16, BITS_2_TO_8, 1e-3)


def vit_tokens(seed: int = 0, rows: int = 64 * 197, width: int = 768) -> Workload:
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((rows, width), dtype=np.float32)
    chans = rng.choice(width, size=2, replace=False)
    x[:, chans] *= np.float32(30.0)
    return Workload("vit_tokens_f32", x, "f32", rows, width, 0.15, 8, BITS_2_TO_8, 5e-4)


def llm_prefill(seed: int = 0, rows: int = 8 * 2048, width: int = 4096) -> Workload:
    rng = np.random.default_rng(seed)
    x = _llm_rows(rng, rows, width)
    return Workload("llm_prefill_bf16", x, "bf16", rows, width, 0.10, 8, BITS_2_TO_8, 1e-3)


def ar_decode_step(seed: int = 0, step: int = 0, rows: int = 256, width: int = 8192) -> Workload:
    rng = np.random.default_rng(seed + step)
    x = _llm_rows(rng, rows, width)
    return Workload("ar_decode_bf16", x, "bf16", rows, width, 0.10, 8, BITS_2_TO_8, 1e-3)


CONFIGS = {1: cnn_map, 2: resnet_stage3, 3: vit_tokens, 4: llm_prefill, 5: ar_decode_step}


def make_config(cfg: int, **kw) -> Workload:
    """Workload number ``cfg`` (1..5); keyword arguments shrink it for tests."""
    return CONFIGS[cfg](**kw)


def adversarial_rows(dtype: str, row_len: int, seed: int = 0) -> np.ndarray:
    """Rows that exercise the degenerate cases of the method: all zero, all equal,
    a single non-zero, one sign only, heavy ties, one huge outlier, denormals,
    alternating signs with equal magnitudes, ascending and descending ramps."""
    rng = np.random.default_rng(seed)
    N = row_len
    rows = []
    rows.append(np.zeros(N, np.float32))
    rows.append(np.full(N, 1.5, np.float32))
    r = np.zeros(N, np.float32); r[N // 3] = -2.0; rows.append(r)
    rows.append(np.abs(rng.standard_normal(N, dtype=np.float32)))
    rows.append(-np.abs(rng.standard_normal(N, dtype=np.float32)))
    rows.append(rng.integers(-3, 4, size=N).astype(np.float32) * np.float32(0.25))
    r = rng.standard_normal(N, dtype=np.float32); r[N // 2] = 3.0e4; rows.append(r)
    r = (rng.integers(1, 200, size=N).astype(np.float32) * np.float32(1e-41)); r[::2] *= -1; rows.append(r)
    r = np.ones(N, np.float32); r[1::2] = -1.0; rows.append(r)
    rows.append(np.arange(1, N + 1, dtype=np.float32) / np.float32(N))
    rows.append(-np.arange(N, 0, -1, dtype=np.float32) / np.float32(N))
    r = rng.standard_normal(N, dtype=np.float32); r[rng.random(N) < 0.97] = 0.0; rows.append(r)
    x = np.stack(rows).astype(np.float32)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    return x
