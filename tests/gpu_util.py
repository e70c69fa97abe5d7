"""Helpers of the GPU parity tests: numpy <-> device tensors for the three storage dtypes."""
import numpy as np

import lcma_inputs as inp


def to_device(stored: np.ndarray, dtype: str):
    import torch
    if dtype == "bf16":
        return torch.from_numpy(stored.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(stored).cuda()


def empty_like_c(M: int, N: int, dtype: str, fill=None):
    import torch
    td = {"f32": torch.float32, "bf16": torch.bfloat16, "f16": torch.float16}[dtype]
    if fill is None:
        return torch.empty((M, N), dtype=td, device="cuda")
    return torch.full((M, N), fill, dtype=td, device="cuda")


def to_host_stored(t, dtype: str) -> np.ndarray:
    import torch
    if dtype == "bf16":
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy()


def to_host_f64(t, dtype: str) -> np.ndarray:
    return inp.widen(to_host_stored(t, dtype), dtype)
