"""Helpers for the GPU parity tests: numpy <-> device tensors, announcing each case."""
import sys

import numpy as np
import torch


def announce(msg):
    """Name the case about to touch the GPU, flushed, so a fault can be attributed."""
    print("[gpu-case] " + msg, file=sys.stderr, flush=True)


def dev(a, dtype=None):
    """numpy -> cuda tensor; uint16 arrays are bf16 bit patterns."""
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint16:
        return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
    if a.dtype == np.uint64:
        return torch.from_numpy(a.view(np.int64)).cuda()
    return torch.from_numpy(a).cuda()


def host(t):
    """cuda tensor -> numpy; bf16 comes back as uint16 bit patterns."""
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).cpu().numpy().view(np.uint16)
    return t.cpu().numpy()


def mask_bits_u64(t):
    return t.cpu().numpy().view(np.uint64)
