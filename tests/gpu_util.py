"""Helpers for the GPU parity tests: numpy <-> device tensors, library handle."""
import numpy as np
import torch


def have_gpu() -> bool:
    return torch.cuda.is_available()


def to_dev(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def words(t: torch.Tensor) -> np.ndarray:
    """Packed-bit device tensor (int32) -> numpy uint32."""
    return t.cpu().numpy().view(np.uint32)


def host(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy()
