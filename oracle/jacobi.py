"""Brute-force cyclic Jacobi eigen-solver for small symmetric matrices
(TEST INFRASTRUCTURE ONLY).  Used to pin the refreshed basis: repeated
Power(A, Q) on a fixed symmetric positive definite A must converge to the
eigenvectors this routine returns, in descending-eigenvalue order and up to
sign (Section 3.2: power iteration followed by QR "to compute eigenvectors").
"""
from __future__ import annotations

import math

import numpy as np


def jacobi_eigh(A, sweeps: int = 60, tol: float = 1e-30):
    """Eigen-decomposition of a symmetric matrix by plane rotations.
    Returns (eigenvalues descending, eigenvectors as columns)."""
    A = np.array(A, dtype=np.float64, copy=True)
    n = A.shape[0]
    V = np.eye(n)
    for _ in range(sweeps):
        off = 0.0
        for p in range(n - 1):
            for q in range(p + 1, n):
                off += A[p, q] * A[p, q]
        if off <= tol:
            break
        for p in range(n - 1):
            for q in range(p + 1, n):
                if A[p, q] == 0.0:
                    continue
                theta = (A[q, q] - A[p, p]) / (2.0 * A[p, q])
                t = math.copysign(1.0, theta) / (abs(theta) + math.sqrt(theta * theta + 1.0))
                c = 1.0 / math.sqrt(t * t + 1.0)
                s = t * c
                for k in range(n):          # A <- A J  (columns p, q)
                    akp, akq = A[k, p], A[k, q]
                    A[k, p] = c * akp - s * akq
                    A[k, q] = s * akp + c * akq
                for k in range(n):          # A <- J^T A  (rows p, q)
                    apk, aqk = A[p, k], A[q, k]
                    A[p, k] = c * apk - s * aqk
                    A[q, k] = s * apk + c * aqk
                for k in range(n):          # V <- V J
                    vkp, vkq = V[k, p], V[k, q]
                    V[k, p] = c * vkp - s * vkq
                    V[k, q] = s * vkp + c * vkq
    w = np.diag(A).copy()
    order = np.argsort(-w, kind="stable")
    return w[order], V[:, order]
