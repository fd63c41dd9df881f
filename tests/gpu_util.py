"""Helpers shared by the GPU parity tests: host arrays <-> device tensors."""
import numpy as np
import torch


def to_device(a: np.ndarray) -> torch.Tensor:
    """fp32 array -> float32 tensor; uint16 (bf16 bit patterns) -> bfloat16 tensor, on cuda:0."""
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).to("cuda:0")
    return torch.from_numpy(a).to("cuda:0")


def to_host(t: torch.Tensor) -> np.ndarray:
    """Inverse of to_device (bf16 comes back as uint16 bit patterns)."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()
