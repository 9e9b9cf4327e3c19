"""Moving 16-bit bit patterns between numpy and torch device tensors (plumbing only)."""
from __future__ import annotations

import numpy as np


def bits_to_device(bits: np.ndarray, dtype: str, device="cuda:0"):
    """uint16 bit patterns [..] -> torch float16 / bfloat16 tensor on the device, same bits."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16))
    t = t.view(torch.float16 if dtype == "f16" else torch.bfloat16)
    return t.to(device)
