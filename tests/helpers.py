"""Small conversions shared by the tests (no method arithmetic)."""
import numpy as np
import torch


def to_oracle_array(t: torch.Tensor) -> np.ndarray:
    """torch fp32 -> float32 ndarray; torch bf16 -> uint16 ndarray of the same bits."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    assert t.dtype == torch.float32
    return t.numpy()
