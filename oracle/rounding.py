"""Oracle: rounding of fp64 results to the storage type (test infrastructure).

Activations and pre-processed pixels are stored in fp32, fp16 or bf16; the
oracle evaluates each stage in fp64 and rounds once (nearest-even) where the
path stores a tensor.  Values are returned widened to fp32 (exact).
"""
from __future__ import annotations

import numpy as np


def round_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f32":
        return x.astype(np.float32)
    if dtype == "f16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        # fp64 -> fp32 -> bf16 would round twice; resolve the fp32-level ties from the fp64 residual.
        r32 = x.astype(np.float32)
        u = r32.view(np.uint32).astype(np.uint64)
        low = u & 0xFFFF
        odd = (u >> 16) & 1
        tie = low == 0x8000
        up = (low > 0x8000) | (tie & (odd == 1))
        resid = np.abs(x) - np.abs(r32.astype(np.float64))
        up = np.where(tie & (resid > 0), True, np.where(tie & (resid < 0), False, up))
        out = (((u >> 16) + up.astype(np.uint64)) << 16).astype(np.uint32)
        res = out.view(np.float32).reshape(r32.shape)
        return np.where(np.isfinite(r32), res, r32)
    raise ValueError(dtype)
