"""Helpers for the GPU tests: numpy <-> device tensors without changing a bit."""
import numpy as np
import torch


def dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def host(t: torch.Tensor, like: np.dtype) -> np.ndarray:
    a = t.detach().cpu().numpy()
    return a.view(np.uint16) if np.dtype(like) == np.uint16 else a


def same_bits(a: np.ndarray, b: np.ndarray) -> bool:
    a, b = np.ascontiguousarray(a), np.ascontiguousarray(b)
    if a.shape != b.shape or a.dtype.itemsize != b.dtype.itemsize:
        return False
    return np.array_equal(a.view(np.uint8), b.view(np.uint8))
