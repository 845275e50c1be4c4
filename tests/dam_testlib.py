"""Shared helpers of the GPU parity tests: packing oracle results into the ABI's layouts and
moving workload arrays to the device. No method arithmetic lives here."""
from __future__ import annotations

import numpy as np
import torch


def pack_rows_u64(m: np.ndarray) -> np.ndarray:
    """[..., n] 0/1 bytes -> [..., ceil(n/64)] u64 words, bit (j % 64) of word j // 64."""
    n = m.shape[-1]
    pad = (-n) % 64
    if pad:
        m = np.concatenate([m, np.zeros(m.shape[:-1] + (pad,), m.dtype)], -1)
    b = np.packbits(m.astype(np.uint8), axis=-1, bitorder="little")
    return np.ascontiguousarray(b).view(np.uint64)


def u64(t: torch.Tensor) -> np.ndarray:
    """int64 device tensor holding u64 bit patterns -> numpy uint64."""
    return t.cpu().numpy().view(np.uint64)


def dev(x: np.ndarray, dtype: str = "f32") -> torch.Tensor:
    """fp32 numpy array of storage-rounded values -> device tensor of the storage dtype."""
    t = torch.from_numpy(np.ascontiguousarray(x))
    if dtype == "bf16":
        t = t.to(torch.bfloat16)
    return t.cuda()


def sync_ok():
    torch.cuda.synchronize()
