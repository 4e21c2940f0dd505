"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def words(t):
    """Packed int32 tensor -> uint32 numpy."""
    return host(t).view(np.uint32)


def gpu_available():
    return torch.cuda.is_available()
