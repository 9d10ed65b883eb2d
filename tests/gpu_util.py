"""Helpers of the GPU parity tests: host <-> device marshalling (no method arithmetic)."""
import numpy as np
import torch


def tdtype(name):
    return torch.bfloat16 if name == "bf16" else torch.float32


def to_dev(a, dtype_name=None):
    """float32 numpy (holding exactly representable values) -> device tensor."""
    t = torch.from_numpy(np.ascontiguousarray(a)).cuda()
    if dtype_name == "bf16":
        t = t.to(torch.bfloat16)
    return t.contiguous()


def to_np(t):
    return t.detach().to(torch.float32).cpu().numpy() if t.is_floating_point() else t.detach().cpu().numpy()


def say(*a):
    print(*a, flush=True)
