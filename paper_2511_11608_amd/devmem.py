"""numpy <-> device tensors for the codec's two element types (bf16 travels as uint16 bit patterns)."""
from __future__ import annotations

import numpy as np
import torch


def to_device(x: np.ndarray, dtype: str) -> torch.Tensor:
    if dtype == "f32":
        return torch.from_numpy(np.ascontiguousarray(x)).cuda()
    return torch.from_numpy(np.ascontiguousarray(x).view(np.int16)).cuda().view(torch.bfloat16)


def to_host(y: torch.Tensor) -> np.ndarray:
    if y.dtype == torch.bfloat16:
        return y.view(torch.int16).cpu().numpy().view(np.uint16)
    return y.cpu().numpy()
