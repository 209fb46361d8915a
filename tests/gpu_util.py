"""Helpers for the GPU parity tests: move seeded numpy inputs to the device, call the library
through its C ABI binding, bring results back."""
import numpy as np

FP32_TOL = 1e-5   # max |gpu - oracle| / sum|terms| for float32 operands (fp32 accumulation)
BF16_TOL = 1e-2   # same metric for bfloat16 operands


def torch_mod():
    import torch
    return torch


def dev(a):
    torch = torch_mod()
    return None if a is None else torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch_mod().cuda.synchronize()
    return t.cpu().numpy()


def sample_indices(total, count, seed):
    """count distinct-ish flat indices in [0, total) including the first and last elements."""
    from synth import rng
    r = rng._raw(seed, 77, count)
    idx = (r % np.uint64(total)).astype(np.int64)
    idx[0], idx[-1] = 0, total - 1
    return idx
