"""Helpers for the GPU parity tests: host <-> device tensors in the oracle's conventions."""
import numpy as np
import torch

DEV = "cuda:0"


def to_dev(a: np.ndarray) -> torch.Tensor:
    """float32 -> float32 tensor; uint16 (bf16 bits) -> bfloat16 tensor."""
    if a.dtype == np.float32:
        return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    assert a.dtype == np.uint16
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).to(DEV).view(torch.bfloat16)


def to_host(t: torch.Tensor) -> np.ndarray:
    """inverse of to_dev; int16 metadata comes back as uint16"""
    t = t.contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    if t.dtype == torch.int16:
        return t.cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def first_mismatch(a: np.ndarray, b: np.ndarray):
    ne = np.argwhere(a != b)
    return None if len(ne) == 0 else tuple(int(v) for v in ne[0])
