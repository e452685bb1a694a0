"""Helpers shared by the GPU parity tests: host arrays -> device tensors and back."""
import numpy as np
import torch

from paper_2402_13485_amd import synth


from paper_2402_13485_amd.binding import to_device as to_dev, to_host  # noqa: E402,F401


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
