"""Upload of generated inputs to the GPU (torch is used for device memory only)."""
import numpy as np
import torch

from .generate import f32_to_bf16_bits


def to_device(x: np.ndarray, dtype: str) -> torch.Tensor:
    """numpy float32 (already storage-rounded) -> GPU tensor of the storage dtype ("f32" or "bf16")."""
    if dtype == "bf16":
        bits = f32_to_bf16_bits(x).view(np.int16)
        return torch.from_numpy(bits).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()


def dev_i32(x) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).cuda()


def dev_i64(x) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.int64)).cuda()


def dev_f32(x) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda()
