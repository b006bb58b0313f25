"""Helpers for the GPU parity tests."""
import numpy as np
import torch


def dev(a: np.ndarray) -> torch.Tensor:
    if a.dtype == np.uint16:  # torch has limited uint16 support: move the bits, then name the type
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.uint16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy()
