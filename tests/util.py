"""Helpers shared by the GPU parity tests (no arithmetic of the method in here)."""
from __future__ import annotations

import os

import numpy as np

THREADS = min(16, os.cpu_count() or 1)

# Parity gates against the fp64 oracle, max-norm relative error per tensor:
#   ||a - ref||_inf / ||ref||_inf
# x and dL/dy: 1e-4; dL/dw: 1e-3 (fp32 arithmetic on the GPU side).
TOL_ACT = 1e-4
TOL_DW = 1e-3


def rel_err(a, ref) -> float:
    a = np.asarray(a, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    denom = np.abs(ref).max()
    if denom == 0.0:
        return float(np.abs(a).max())
    return float(np.abs(a - ref).max() / denom)


def elementwise_ok(a, ref, rtol) -> bool:
    """|a - ref| <= atol + rtol |ref| with atol = rtol * 1e-2 * ||ref||_inf."""
    a = np.asarray(a, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    atol = rtol * 1e-2 * np.abs(ref).max()
    return bool(np.all(np.abs(a - ref) <= atol + rtol * np.abs(ref)))


def dev(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()


def host(t):
    return t.detach().cpu().numpy()
