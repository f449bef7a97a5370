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


def rel_err(got, ref, floor: str = "tensor") -> float:
    """max_i |got_i - ref_i| / max(|ref_i|, s_i): element-wise relative error with a floor s_i, so that elements
    near zero do not blow it up.  s_i is the RMS of ref over the slice element i belongs to:
      floor="tensor": the whole tensor (homogeneous tensors: weights' gradients of one matrix, [T,k] arrays)
      floor="row":    the last-dimension row (token rows of activations and their gradients, whose scale follows
                      the token's combine weight and therefore differs by orders of magnitude between rows)
      floor="expert": one expert's matrix of an [E, ., .] tensor (its scale follows the expert's row count)
    Rounding a stored intermediate to bf16 perturbs a dot product by about 2^-9 times the 2-norm of its terms,
    which is the scale of the row (or matrix), not of the individual output element; see
    tests/test_tolerance_model.py for the arithmetic."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    if floor == "tensor" or ref.ndim == 1:
        s = np.sqrt(np.mean(ref * ref))
    elif floor == "row":
        s = np.sqrt(np.mean(ref * ref, axis=-1, keepdims=True))
    elif floor == "expert":
        s = np.sqrt(np.mean(ref * ref, axis=tuple(range(1, ref.ndim)), keepdims=True))
    else:
        raise ValueError(floor)
    denom = np.maximum(np.abs(ref), s)
    diff = np.abs(got - ref)
    # a slice that is exactly zero in the reference must be exactly zero in the result
    zero = denom == 0.0
    if np.any(diff[np.broadcast_to(zero, diff.shape)] != 0.0):
        return float("inf")
    return float((diff / np.where(zero, 1.0, denom)).max())


def rel_err_fro(got, ref) -> float:
    """||got - ref||_F / ||ref||_F over the whole tensor."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    n = float(np.sqrt((ref * ref).sum()))
    e = float(np.sqrt(((got - ref) ** 2).sum()))
    return e / n if n > 0 else (0.0 if e == 0 else float("inf"))


def rel_err_norm(got, ref) -> float:
    """max over last-dimension rows of ||got_r - ref_r||_2 / ||ref_r||_2: the relative error of each output
    vector (a token's row, a row of a weight-gradient matrix).  A row that is exactly zero in the reference must
    be exactly zero in the result."""
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    n = np.sqrt((ref * ref).sum(axis=-1))
    e = np.sqrt(((got - ref) ** 2).sum(axis=-1))
    if np.any(e[n == 0.0] != 0.0):
        return float("inf")
    return float((e / np.where(n == 0.0, 1.0, n)).max())


def assert_close_chain(got, ref, dtype_name: str, what: str, floor: str = "row", norm: str = "row"):
    """Criterion for outputs at the end of the whole layer, where a chain of bf16-stored intermediates (G, U, A,
    Y, dY, dG, dU, ...) separates the result from the unrounded float64 oracle: the relative error of every output
    row in the 2-norm must be within the stated tolerance, and no single element may be off by more than 4x the
    tolerance relative to max(|ref|, slice RMS) (an implementation with exact accumulation already reaches 3.6e-2
    on that element-wise figure for bf16; see tests/test_tolerance_model.py).  float32 workloads keep the strict
    element-wise bound."""
    assert np.isfinite(np.asarray(got, np.float64)).all(), f"{what}: non-finite values"
    # norm="tensor" is for the gate weights' gradient only: softmax backward subtracts sum_e p*dp from dp, which
    # amplifies the bf16 error carried by dw = <dOut, Y> by up to 1/(1 - p_max); with skewed routing p_max -> 1,
    # so single rows of dW_router (E entries each) are ill-conditioned and only the tensor as a whole is compared
    # in the 2-norm.
    en = rel_err_norm(got, ref) if norm == "row" else rel_err_fro(got, ref)
    ee = rel_err(got, ref, floor)
    tol = TOL[dtype_name]
    assert en <= tol, f"{what}: max row-wise relative error {en:.3e} > {tol:.1e}"
    cap = tol if dtype_name == "f32" else 4 * tol
    assert ee <= cap, f"{what}: max element-wise relative error {ee:.3e} > {cap:.1e}"
    return en, ee


def assert_close(got, ref, dtype_name: str, what: str, scale: float = 1.0, floor: str = "tensor"):
    e = rel_err(got, ref, floor)
    assert np.isfinite(np.asarray(got, np.float64)).all(), f"{what}: non-finite values"
    assert e <= TOL[dtype_name] * scale, f"{what}: max relative error {e:.3e} > {TOL[dtype_name] * scale:.1e}"
    return e


def chain_errors_dev(got: torch.Tensor, ref: np.ndarray):
    """(max row-wise 2-norm relative error, max element-wise relative error against max(|ref|, row RMS)) of a
    device tensor against a float64 reference, computed in float64 on the device: the metric of
    assert_close_chain(floor="row", norm="row") for tensors too large to compare on the host in reasonable time
    (one expert's weight gradients at the large shapes).  Only the comparison runs on the device; the reference is
    the oracle's."""
    r = torch.from_numpy(np.ascontiguousarray(ref, dtype=np.float64)).cuda()
    g = got.to(torch.float64)
    assert g.shape == r.shape, (tuple(g.shape), tuple(r.shape))
    if r.numel() == 0:
        return 0.0, 0.0
    assert torch.isfinite(g).all(), "non-finite values"
    diff = g - r
    n = r.pow(2).sum(dim=-1).sqrt()
    e = diff.pow(2).sum(dim=-1).sqrt()
    if bool((e[n == 0] != 0).any()):
        return float("inf"), float("inf")
    en = float((e / torch.where(n == 0, torch.ones_like(n), n)).max())
    s_ = r.pow(2).mean(dim=-1, keepdim=True).sqrt()
    den = torch.maximum(r.abs(), s_)
    ee = float((diff.abs() / torch.where(den == 0, torch.ones_like(den), den)).max())
    return en, ee


def assert_close_chain_dev(got: torch.Tensor, ref: np.ndarray, dtype_name: str, what: str):
    """assert_close_chain(floor="row", norm="row") with the comparison done on the device."""
    en, ee = chain_errors_dev(got, ref)
    tol = TOL[dtype_name]
    cap = tol if dtype_name == "f32" else 4 * tol
    assert en <= tol, f"{what}: max row-wise relative error {en:.3e} > {tol:.1e}"
    assert ee <= cap, f"{what}: max element-wise relative error {ee:.3e} > {cap:.1e}"
    return en, ee
