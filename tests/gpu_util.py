"""Helpers for the GPU parity tests (tensor transfer, context and key setup)."""
import numpy as np
import torch


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint64)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


def zeros(*shape):
    return torch.zeros(shape, dtype=torch.uint64, device="cuda")
