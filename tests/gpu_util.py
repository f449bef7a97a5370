"""Helpers shared by the GPU parity tests: host<->device conversion and the error metric."""
from __future__ import annotations

import numpy as np
import torch

# tolerances of the benchmark definition: max relative error, float32 workloads / bf16 workloads
TOL = {"f32": 1e-5, "bf16": 2e-2}


def torch_dtype(name: str) -> torch.dtype:
    return torch.float32 if name == "f32" else torch.bfloat16


def to_dev(a, dtype_name: str) -> torch.Tensor:
    """float32 numpy array holding storage-exact values -> device tensor of the storage type (exact)."""
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32))
    return t.to(torch_dtype(dtype_name)).cuda().contiguous()


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel_err(got, ref) -> float:
    """max_i |got_i - ref_i| / max(|ref_i|, rms(ref)): element-wise relative error, floored at the tensor's RMS
    so that elements near zero do not blow it up."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    rms = float(np.sqrt(np.mean(ref * ref)))
    if rms == 0.0:
        return float(np.abs(got).max())
    return float((np.abs(got - ref) / np.maximum(np.abs(ref), rms)).max())


def assert_close(got, ref, dtype_name: str, what: str, scale: float = 1.0):
    e = rel_err(got, ref)
    assert np.isfinite(np.asarray(got, np.float64)).all(), f"{what}: non-finite values"
    assert e <= TOL[dtype_name] * scale, f"{what}: max relative error {e:.3e} > {TOL[dtype_name] * scale:.1e}"
    return e
