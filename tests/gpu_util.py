"""Helpers for the GPU parity tests: numpy <-> torch device tensors (bf16 travels as uint16
bit patterns on the numpy side)."""
import numpy as np
import torch


def to_dev(a):
    """float32 array -> float32 cuda tensor; uint16 array -> bfloat16 cuda tensor (same bits);
    uint8 -> uint8."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(a).cuda()


def to_host(t):
    """cuda tensor -> numpy (bfloat16 comes back as uint16 bit patterns)."""
    t = t.detach().contiguous().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def sync():
    torch.cuda.synchronize()
