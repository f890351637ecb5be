"""Helpers shared by the tests: tensor <-> bf16 bit-pattern conversions and the
comparison rules used for parity."""
import numpy as np
import torch


def bits(t: torch.Tensor) -> np.ndarray:
    """bf16 tensor (any device) -> uint16 numpy array of its bit patterns."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.uint16).numpy()


def weights_bits(w: dict) -> dict:
    return {k: ([bits(a) for a in v] if isinstance(v, list) else bits(v)) for k, v in w.items()}


def from_bits(a: np.ndarray, device="cpu") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).view(torch.bfloat16).to(device)
