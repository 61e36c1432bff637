"""Helpers of the GPU parity tests (not collected by pytest)."""
import sys

import numpy as np
import torch


def say(*parts):
    """Name the case on stdout before the GPU step that runs it."""
    print("[gpu-case]", *parts, flush=True)


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.detach().cpu().numpy()


def same_bits(a, b):
    """fp32 arrays identical bit for bit (0 ulp)."""
    a = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    b = np.ascontiguousarray(b, dtype=np.float32).view(np.uint32)
    return a.shape == b.shape and np.array_equal(a, b)
