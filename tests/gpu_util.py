"""Helpers of the GPU parity tests: device upload / download through torch (memory only)."""
import numpy as np
import torch


def dev(a):
    """numpy -> device tensor; uint16 (bfloat16 bits) travels as int16."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda()
    return torch.from_numpy(a).cuda()


def host(t, like=None):
    a = t.cpu().numpy()
    if a.dtype == np.int16:
        a = a.view(np.uint16)
    return a


def empty(shape, dtype=torch.float32):
    return torch.empty(shape, dtype=dtype, device="cuda")
