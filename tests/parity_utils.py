"""Tolerance helpers shared by the GPU parity tests."""
import numpy as np


def rel_errs(a, b):
    """(max-norm relative error, l2 relative error) of a against reference b."""
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    if b.size == 0:
        return 0.0, 0.0
    den_m = max(np.abs(b).max(), 1e-30)
    den_2 = max(np.linalg.norm(b.ravel()), 1e-30)
    return np.abs(a - b).max() / den_m, np.linalg.norm((a - b).ravel()) / den_2


def assert_close(a, b, tol, what=""):
    """Per tensor: max|a-b| / max|b| <= tol and ||a-b||_2 / ||b||_2 <= tol."""
    assert np.isfinite(np.asarray(a, np.float64)).all(), f"{what}: non-finite values"
    em, e2 = rel_errs(a, b)
    assert em <= tol and e2 <= tol, f"{what}: max-rel {em:.3e}, l2-rel {e2:.3e} > {tol}"


def bf16_round(x):
    """Round-to-nearest-even float32 -> bfloat16 -> float32 (numpy only)."""
    u = np.asarray(x, np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32)
