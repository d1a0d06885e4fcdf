"""Helpers for the GPU parity tests: moving bf16 bit patterns to and from the device."""
import numpy as np
import torch

import workloads as wl


def to_dev(a) -> torch.Tensor:
    """BF16Array (or uint16 bits) -> bfloat16 tensor on the GPU with the same bits."""
    bits = a.bits if isinstance(a, wl.BF16Array) else a
    t = torch.from_numpy(np.ascontiguousarray(bits).view(np.int16).copy())
    return t.view(torch.bfloat16).cuda()


def f32_to_dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def from_dev(t: torch.Tensor) -> np.ndarray:
    """Device tensor -> float32 numpy (bf16 widened exactly)."""
    t = t.detach().cpu().contiguous()
    if t.dtype == torch.bfloat16:
        return wl.bf16_bits_to_f32(t.view(torch.int16).numpy().view(np.uint16))
    return t.numpy().astype(np.float32, copy=False)


def bits_from_dev(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
