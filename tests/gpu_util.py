"""Helpers shared by the GPU parity tests: host arrays -> device tensors and back."""
import numpy as np
import torch

from paper_2402_13485_amd import synth


def to_dev(a: np.ndarray) -> torch.Tensor:
    """numpy -> cuda tensor; uint16 arrays are bf16 bit patterns, uint64 travel as int64."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).cuda()
    return torch.from_numpy(a).cuda()


def to_host(t: torch.Tensor) -> np.ndarray:
    """cuda tensor -> numpy; bf16 comes back as uint16 bit patterns."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def host_f64(t: torch.Tensor) -> np.ndarray:
    h = to_host(t)
    return synth.as_float(h).astype(np.float64)


def u64(t: torch.Tensor) -> np.ndarray:
    return t.cpu().numpy().view(np.uint64)


def sentinel_like(a: np.ndarray) -> np.ndarray:
    """A recognisable bit pattern for 'must not be written' checks."""
    if a.dtype == np.uint16:
        return np.full_like(a, 0x4D4D)
    if a.dtype == np.float32:
        return np.full_like(a, 12345.5)
    return np.full_like(a, -77)
