"""Comparison metrics used by the tests (TEST INFRASTRUCTURE ONLY)."""
from __future__ import annotations

import numpy as np


def rel_err(a, b) -> float:
    """max|a - b| / max|b|: one number per tensor.  Element-wise relative error is
    meaningless next to zeros, so the error is scaled by the tensor's largest entry."""
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    if a.shape != b.shape:
        raise ValueError(f"shape mismatch {a.shape} vs {b.shape}")
    if a.size == 0:
        return 0.0
    if not (np.isfinite(a).all() and np.isfinite(b).all()):
        return float("inf")
    scale = np.abs(b).max()
    diff = np.abs(a - b).max()
    return float(diff / scale) if scale > 0 else float(diff)


def one_one_norm(A) -> float:
    """(1,1)-norm: the sum of absolute values of all entries (Section 2.3)."""
    return float(np.abs(np.asarray(A, dtype=np.float64)).sum())


def misalignment(Q, H) -> float:
    """||Q^T H Q||_(1,1) / tr(H): 1 when Q diagonalises the PSD matrix H,
    larger otherwise (the misalignment proxy of Section 2.3 applied to one
    Kronecker factor; the product over factors is the norm of the whole
    Hessian by the Kronecker (1,1)-norm lemma of the misalignment appendix)."""
    Q = np.asarray(Q, dtype=np.float64)
    H = np.asarray(H, dtype=np.float64)
    return one_one_norm(Q.T @ H @ Q) / float(np.trace(H))


def orthogonality_defect(Q) -> float:
    Q = np.asarray(Q, dtype=np.float64)
    return float(np.abs(Q.T @ Q - np.eye(Q.shape[1])).max())
