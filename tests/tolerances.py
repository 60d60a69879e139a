"""Tolerance terms that the GPU parity tests add to the stated bars, in one place, so that the CPU
tests (tests/test_tolerance_models.py) can show on the host, with the oracle and float32 numpy only,
that each term has the size the arithmetic gives it."""
import numpy as np

TOL = 1e-4

# Multiple of cond(A) * 2^-24 allowed on top of 1e-4 where a basis comes from ill-conditioned
# statistics (the 512 x 128 quadratic).  Worst measured on the GPU: 0.66 (left basis, step 500).
QUAD_COND_FACTOR = 1.25

# Multiples of the per-sigma term of `young_moment_floor` allowed where Adam's quotient amplifies the FP32
# rounding of the rotated gradient (refresh-every-step configuration).  Measured: the GPU's worst error there is
# 1.79e-4 = 1e-4 + 1.1 of that term; a float32 product on the host moves the quotient by 1.1 of it as well
# (tests/test_tolerance_models.py).  3.5 keeps the whole allowance below twice the measured worst.
YOUNG_MOMENT_SIGMAS = 3.5


def lapack_qr(P):
    """LAPACK's QR with the oracle's sign convention diag(R) >= 0 (the orthogonal factor of a
    full-rank matrix is unique; pinned against the oracle's own Householder loop on the CPU)."""
    q, r = np.linalg.qr(P)
    d = np.where(np.diag(r) < 0, -1.0, 1.0)
    return q * d[None, :], r * d[:, None]


def storage_floor(W, dW):
    """Weights are stored in FP32, so an update read back as a difference of stored weights is known
    only to one ulp of W: 2^-23 max|W| / max|dW| relative to the update."""
    s = np.abs(dW).max()
    return float(2.0 ** -23 * np.abs(W).max() / s) if s > 0 else 0.0


def young_moment_floor(hp, G, sigmas=YOUNG_MOMENT_SIGMAS):
    """While the second moment holds one sample (first step, or a basis refreshed every step), the
    quotient m / sqrt(s + eps) = (1 - beta1) g / sqrt((1 - beta2) g^2 + eps) has slope (1 - beta1) / sqrt(eps)
    at entries whose rotated gradient is near zero, so the FP32 rounding of a rotated-gradient entry (a
    length-K dot product: about 2^-24 times the row norm of G as a standard deviation) is amplified by that
    slope.  Relative to max|X| = (1 - beta1) / sqrt(1 - beta2) this is
    2^-24 * max_row_norm(G) * sqrt(1 - beta2) / sqrt(eps) per standard deviation."""
    row = float(np.sqrt((np.asarray(G, dtype=np.float64) ** 2).sum(axis=1)).max())
    return sigmas * 2.0 ** -24 * row * np.sqrt(1.0 - hp.beta2) / np.sqrt(hp.eps)
