"""Error measures used by the parity tests."""
import numpy as np


def rel_frobenius(got, want):
    """||got - want||_F / ||want||_F in fp64 (0 when both are all-zero)."""
    g = np.asarray(got, dtype=np.float64)
    w = np.asarray(want, dtype=np.float64)
    if g.shape != w.shape:
        raise ValueError(f"shape mismatch {g.shape} vs {w.shape}")
    den = np.linalg.norm(w.ravel())
    num = np.linalg.norm((g - w).ravel())
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return float(num / den)
