"""Helpers for the GPU parity tests: host <-> device transfers of raw bf16 / uint32 arrays."""
import numpy as np
import torch

import salr_workloads as wl


def dev():
    return torch.device("cuda:0")


def to_dev_u16(a: np.ndarray) -> torch.Tensor:
    """uint16 patterns -> int16 CUDA tensor whose storage is padded to a multiple of 16 bytes."""
    a = np.ascontiguousarray(a, dtype=np.uint16)
    flat = a.reshape(-1)
    padded = max(8, (flat.size + 7) // 8 * 8)
    buf = torch.zeros(padded, dtype=torch.int16, device=dev())
    if flat.size:
        buf[:flat.size] = torch.from_numpy(flat.view(np.int16)).to(dev())
    return buf[:flat.size].view(a.shape) if flat.size else buf[:0].view(a.shape)


def to_dev_u32(a: np.ndarray) -> torch.Tensor:
    a = np.ascontiguousarray(a, dtype=np.uint32)
    return torch.from_numpy(a.view(np.int32)).to(dev())


def to_host_u16(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().numpy().view(np.uint16)


def to_host_u32(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().contiguous().numpy().view(np.uint32)


def y_to_f64(t: torch.Tensor) -> np.ndarray:
    return wl.bf16_bits_to_f32(to_host_u16(t)).astype(np.float64)
