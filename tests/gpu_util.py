"""Helpers shared by the GPU parity tests: host <-> device plumbing only."""
import numpy as np
import torch


def to_dev(a: np.ndarray) -> torch.Tensor:
    """float32 array -> float32 device tensor; uint16 array of bf16 bits -> bf16
    device tensor; uint8 -> uint8."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).view(torch.bfloat16).cuda()
    return torch.from_numpy(a).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def same_floats(a: np.ndarray, b: np.ndarray) -> bool:
    """Bit equality of float32 arrays (or bf16 bit arrays), any NaN equal to any NaN."""
    if a.dtype == np.uint16:
        na, nb = (a & 0x7FFF) > 0x7F80, (b & 0x7FFF) > 0x7F80
        return bool(np.array_equal(na, nb) and np.array_equal(a[~na], b[~nb]))
    na, nb = np.isnan(a), np.isnan(b)
    return bool(np.array_equal(na, nb) and np.array_equal(a[~na].view(np.uint32), b[~nb].view(np.uint32)))
