"""Tolerance check shared by the GPU parity tests.

fp32 path: per tensor, max|a-b| <= tol * max|b| and ||a-b||_2 <= tol * ||b||_2 with
tol = 1e-4 (the tolerance the target states for fp32); 2e-2 for bf16 inputs.
"""
import numpy as np

TOL_F32 = 1e-4
TOL_BF16 = 2e-2


def check(got, want, tol, what):
    got = np.asarray(got.detach().cpu().numpy() if hasattr(got, "detach") else got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (what, got.shape, want.shape)
    assert np.isfinite(got).all(), f"{what}: non-finite values"
    if want.size == 0:
        return 0.0
    scale = max(np.abs(want).max(), 1e-30)
    e_max = np.abs(got - want).max() / scale
    e_l2 = np.linalg.norm(got - want) / max(np.linalg.norm(want), 1e-30)
    assert e_max <= tol and e_l2 <= tol, f"{what}: max err {e_max:.3e}, l2 err {e_l2:.3e} > {tol}"
    return e_max
