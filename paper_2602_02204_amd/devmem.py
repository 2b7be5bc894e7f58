"""Host arrays <-> device tensors for callers that use PyTorch for device memory (argument marshalling only)."""
from __future__ import annotations

import numpy as np
import torch


def to_dev(a: np.ndarray, dtype: str | None = None):
    """Host array -> device tensor; bf16 bit patterns (uint16) are reinterpreted, not converted."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def bits_of(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> host numpy with the stored bits (bf16 comes back as uint16)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()
