"""Helpers for the GPU parity tests: host <-> device conversion and the error metric."""
import numpy as np
import torch

import workloads as W
from oracle import layer as L

DEV = "cuda:0"


def tdtype(dtype):
    return {W.FP32: torch.float32, W.FP16: torch.float16}.get(dtype, torch.bfloat16)


def to_dev(a, dtype):
    """numpy array (values already representable in the storage type) -> device tensor."""
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(DEV).to(tdtype(dtype)).contiguous()


def to_np(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def store(a, dtype):
    """Round host values to the storage type (returns fp32 numpy)."""
    a = np.asarray(a, dtype=np.float32)
    if dtype == W.FP16:
        return a.astype(np.float16).astype(np.float32)
    return W.round_to_bf16(a) if dtype == W.BF16 else a


def err(got, ref):
    return L.max_rel_err(to_np(got) if isinstance(got, torch.Tensor) else got, ref)


# fp16 keeps 3 more mantissa bits than bf16 (2^-11 against 2^-8 per rounding): an eighth of the bf16 bar, doubled
TOL = {W.FP32: 1e-4, W.BF16: 2e-2, W.FP16: 2.5e-3}
