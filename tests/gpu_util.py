"""Helpers shared by the GPU parity tests (marshalling only)."""
import numpy as np
import torch


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    return t.cpu().numpy()


def rand_codes(rng, shape, bits):
    m = (1 << bits) - 1
    v = 2 * rng.integers(0, 1 << bits, size=shape) - m
    return v.astype(np.int8 if bits <= 7 else np.int16)


def planes_u32(t):
    """GPU int32 plane tensor -> numpy uint32."""
    return host(t).view(np.uint32)


def say(*a):
    print(*a, flush=True)
