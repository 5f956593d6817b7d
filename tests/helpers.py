"""Shared plumbing of the GPU parity tests (host<->device copies, comparisons)."""
import numpy as np
import torch

from fs_workloads.checks import (ATOL, RTOL, assert_bf16_within_1ulp, assert_close_f32,  # noqa: F401
                                 assert_rows_close, bf16_beyond_1ulp)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def table_to_dev(w: np.ndarray) -> torch.Tensor:
    """float32 array -> fp32 tensor; uint16 array of bf16 bit patterns -> bf16 tensor."""
    if w.dtype == np.float32:
        return dev(w)
    assert w.dtype == np.uint16
    return dev(w.view(np.int16)).view(torch.bfloat16)


def table_to_host(t: torch.Tensor) -> np.ndarray:
    if t.dtype == torch.float32:
        return t.cpu().numpy()
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def exact_f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """For values that are exactly representable in bf16 (the hash initialiser's)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    assert not np.any(u & np.uint32(0xFFFF)), "value not exact in bf16"
    return (u >> np.uint32(16)).astype(np.uint16)
