"""Helpers shared by the GPU parity tests."""
import numpy as np
import torch

# Tolerances of the parity bar: normalised max error max|a-b| / max|b| per tensor.
TOL = {"f32": 1e-5, "bf16": 2e-2}
TORCH_DT = {"f32": torch.float32, "bf16": torch.bfloat16}


def nerr(got, ref) -> float:
    """Normalised max error of `got` (torch tensor or array) against the oracle's float64 `ref`."""
    if isinstance(got, torch.Tensor):
        got = got.detach().to(torch.float32).cpu().numpy()
    got = np.asarray(got, np.float64)
    ref = np.asarray(ref, np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    if ref.size == 0:
        return 0.0
    assert np.all(np.isfinite(got)), "non-finite values in the GPU result"
    return float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-30))


def dev(a, dtype="f32"):
    """Upload a numpy array to cuda:0 in the given storage dtype (values are already representable)."""
    t = torch.from_numpy(np.ascontiguousarray(a))
    if t.dtype in (torch.float32, torch.float64):
        t = t.to(TORCH_DT[dtype])
    return t.cuda()


def require_gpu():
    import pytest
    if not torch.cuda.is_available():
        pytest.fail("GPU test selected but no GPU is visible")
