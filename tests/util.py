"""Shared helpers for the parity tests."""
import numpy as np

# Tolerances of the parity bar: max-norm relative error per tensor, max|gpu - oracle| / max|oracle|.
TOL_F32 = 1e-4
TOL_BF16 = 2e-2


def rel_err(gpu, ref) -> float:
    gpu = np.asarray(gpu, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert gpu.shape == ref.shape, (gpu.shape, ref.shape)
    denom = float(np.max(np.abs(ref))) if ref.size else 0.0
    num = float(np.max(np.abs(gpu - ref))) if ref.size else 0.0
    if denom == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / denom


def assert_close(gpu, ref, tol, what=""):
    e = rel_err(gpu, ref)
    assert np.all(np.isfinite(np.asarray(gpu, dtype=np.float64))), f"{what}: non-finite values in GPU result"
    assert e <= tol, f"{what}: max-norm relative error {e:.3e} > {tol:.1e}"
    return e


def to_dev(a, device="cuda:0"):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to(device)


def to_np(t):
    import torch
    torch.cuda.synchronize()
    return t.detach().cpu().numpy()
