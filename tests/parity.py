"""Shared helpers for the GPU parity tests: tolerances, the error measure, tensor plumbing."""
import numpy as np
import torch

# Componentwise error relative to the abs-sum scale  sum_j |A^_ij| |x_j|  (propagated through
# the layers), plus the norm-wise error; both must be within the tolerance.
TOL = {"f32": 1e-5, "bf16": 2e-2}


def to_device(arr: np.ndarray, dtype: str) -> torch.Tensor:
    """Input array (float32 values or uint16 bf16 bit patterns) -> cuda tensor."""
    if dtype == "bf16":
        assert arr.dtype == np.uint16
        return torch.from_numpy(arr.view(np.int16).copy()).cuda().view(torch.bfloat16)
    assert arr.dtype == np.float32
    return torch.from_numpy(arr).cuda()


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float64).cpu().numpy()


def errors(got: np.ndarray, ref: np.ndarray, scale: np.ndarray):
    comp = float((np.abs(got - ref) / (scale + 1e-300)).max()) if got.size else 0.0
    norm = float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300)) if got.size else 0.0
    return comp, norm


def assert_close(got, ref, scale, dtype, what=""):
    comp, norm = errors(got, ref, scale)
    tol = TOL[dtype]
    assert comp <= tol and norm <= tol, f"{what}: componentwise {comp:.3e}, normwise {norm:.3e} > {tol}"
    return comp, norm
