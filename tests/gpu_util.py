"""Helpers shared by the GPU tests: upload raw storage words, call the library through its C-ABI
binding, bring the result back as numpy arrays."""
from __future__ import annotations

import numpy as np

F32, F16, BF16 = 0, 1, 2


def to_device(bits: np.ndarray, dtype: int):
    """Raw storage words ([n] or [batch, n]) -> a GPU tensor of the matching floating-point type."""
    import torch
    b = np.ascontiguousarray(bits)
    if dtype == F32:
        return torch.from_numpy(b.view(np.float32)).cuda()
    t = torch.from_numpy(b.view(np.int16)).cuda()
    return t.view(torch.float16 if dtype == F16 else torch.bfloat16)


def values_to_bits(vals, dtype: int) -> np.ndarray:
    import torch
    if dtype == F32:
        return vals.view(torch.int32).cpu().numpy().view(np.uint32)
    return vals.view(torch.int16).cpu().numpy().view(np.uint16)


def gpu_topk(x_dev, dtype: int, k: int, largest: bool = True, scaling: bool = False, seed: int = 0,
             tuning=None, workspace=None, sorted: bool = False):
    """One call through the binding.  Returns (value words [batch,k], int64 indices [batch,k], traces, workspace)."""
    import torch
    from paper_2501_14336_amd import binding as B
    vals, idx, ws = B.topk(x_dev, k, largest, scaling=scaling, seed=seed, tuning=tuning, workspace=workspace, sorted=sorted)
    torch.cuda.synchronize()
    batch = 1 if x_dev.dim() == 1 else x_dev.shape[0]
    traces = B.read_trace(ws, batch)
    return values_to_bits(vals, dtype), idx.cpu().numpy(), traces, ws
