"""Host <-> device marshalling of the scan's element types.

Argument plumbing only: how a numpy array of each element type travels to a torch
device tensor and back (unsigned integers and structs travel as signed 32- or
64-bit words, because torch has no such dtypes).  No arithmetic of the scan, and
nothing of the CPU oracle, lives here; bench.py, the GPU tests and smoke() share it.
"""
from __future__ import annotations

import numpy as np
import torch

from ks_inputs import ARGMAX_DTYPE

_SIGNED_VIEW = {np.dtype(np.uint16): np.int16, np.dtype(np.uint32): np.int32, np.dtype(np.uint64): np.int64}


def to_device(x: np.ndarray, device="cuda") -> torch.Tensor:
    """Copy a host array to the device as raw storage (unsigned and struct types travel as signed ints)."""
    x = np.ascontiguousarray(x)
    if x.dtype == ARGMAX_DTYPE:
        x = x.view(np.int32).reshape(-1, 4)
    elif x.dtype.names:                      # any other struct of 32-bit words
        x = x.view(np.int32).reshape(len(x), x.dtype.itemsize // 4)
    elif x.dtype in _SIGNED_VIEW:
        x = x.view(_SIGNED_VIEW[x.dtype])
    return torch.from_numpy(x).to(device)


def to_host(t: torch.Tensor, like_dtype) -> np.ndarray:
    """Copy a device tensor back and view it as `like_dtype` again."""
    a = t.cpu().numpy()
    like_dtype = np.dtype(like_dtype)
    if like_dtype.names:
        return a.reshape(-1).view(like_dtype)
    if like_dtype in _SIGNED_VIEW:
        return a.view(like_dtype)
    return a
