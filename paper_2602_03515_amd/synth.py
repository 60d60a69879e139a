"""Seeded synthetic inputs for the basis-rotation optimizer step.

This module only MAKES inputs (weights, gradient sequences, a quadratic test
problem).  It holds none of the optimizer's arithmetic, so both the CPU oracle's
tests and the HIP path's tests may draw identical buffers from it.

The inputs stand in for the paper's workload (language-model gradients, Section 4
and the experimental-details appendix): dense-contraction time does not depend on
the data, and parity only needs reproducible, well-conditioned matrices of the
right shapes.  Recipes:

  * `spiked_gradients`  -- G_t = U diag(s) V^T + noise_std * N_t with Haar U, V
    fixed over time and s_i = 1/i (one 256 x 256 matrix, 20 steps).
  * `lowrank_gradients` -- G_t = A diag(s) B^T + sigma * N_t, A, B with 64
    orthonormal columns fixed per matrix, s_i = 1/i, fresh noise each step
    (transformer-layer and pipeline-stage shapes).
  * `QuadraticProblem`  -- f(W) = 1/2 <W - W*, H_L (W - W*) H_R> with
    H_L = V_L diag(lam_L) V_L^T, H_R likewise, eigenvalues log-uniform in
    [1e-3, 1]; gradient H_L (W - W*) H_R + noise_std * N.
  * `fisher_samples`    -- G = H_L^{1/2} Z H_R^{1/2}, Z standard normal, so that
    E[G G^T] = tr(H_R) H_L and E[G^T G] = tr(H_L) H_R (the Kronecker lemma used in
    the proof of Theorem 3.1).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

# Shapes of the benchmark workloads (rows m, columns n), one tuple per weight matrix.
LLAMA_LAYER_2048 = [(2048, 2048)] * 4 + [(2048, 5632)] * 2 + [(5632, 2048)]
STAGE_3B_LAYER = [(2560, 2560)] * 4 + [(2560, 6912)] * 2 + [(6912, 2560)]
STAGE_3B = STAGE_3B_LAYER * 8
EMBEDDING_SHARD = (32000, 2560)


def haar_orthogonal(rng: np.random.Generator, n: int) -> np.ndarray:
    """Haar-distributed orthogonal matrix: QR of a Gaussian, diag(R) made positive."""
    q, r = np.linalg.qr(rng.standard_normal((n, n)))
    return q * np.where(np.diag(r) < 0, -1.0, 1.0)[None, :]


def orthonormal_columns(rng: np.random.Generator, n: int, k: int) -> np.ndarray:
    q, r = np.linalg.qr(rng.standard_normal((n, k)))
    return q * np.where(np.diag(r) < 0, -1.0, 1.0)[None, :]


def to_bf16_f32(x: np.ndarray) -> np.ndarray:
    """Round float values to bfloat16 (nearest even); returned as float32 holding
    exactly representable bfloat16 values."""
    f = np.ascontiguousarray(np.asarray(x, dtype=np.float32))
    b = f.view(np.uint32).astype(np.uint64)
    b = (b + 0x7FFF + ((b >> 16) & 1)) & 0xFFFF0000
    return b.astype(np.uint32).view(np.float32).reshape(f.shape)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """uint16 bit patterns of the bfloat16 rounding of x."""
    return (to_bf16_f32(x).view(np.uint32) >> 16).astype(np.uint16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    return (np.asarray(bits, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def spiked_gradients(seed: int = 0, m: int = 256, n: int = 256, steps: int = 20,
                     noise_std: float = 0.1):
    """Weights W0 ~ N(0, 1) and `steps` gradients U diag(1/i) V^T + noise (float32)."""
    rng = np.random.default_rng(seed)
    k = min(m, n)
    U = haar_orthogonal(rng, m)[:, :k]
    V = haar_orthogonal(rng, n)[:, :k]
    s = 1.0 / np.arange(1, k + 1)
    signal = (U * s[None, :]) @ V.T
    W0 = rng.standard_normal((m, n)).astype(np.float32)
    grads = [(signal + noise_std * rng.standard_normal((m, n))).astype(np.float32)
             for _ in range(steps)]
    return W0, grads


def lowrank_gradients(seed: int, m: int, n: int, steps: int, rank: int = 64,
                      sigma: float = 0.01, bf16: bool = False):
    """W0 ~ N(0, 0.02^2)-like weights and `steps` low-rank-plus-noise gradients."""
    rng = np.random.default_rng(seed)
    rank = min(rank, m, n)
    A = orthonormal_columns(rng, m, rank)
    B = orthonormal_columns(rng, n, rank)
    s = 1.0 / np.arange(1, rank + 1)
    signal = (A * s[None, :]) @ B.T
    W0 = (0.02 * rng.standard_normal((m, n))).astype(np.float32)
    grads = []
    for _ in range(steps):
        g = (signal + sigma * rng.standard_normal((m, n))).astype(np.float32)
        grads.append(to_bf16_f32(g) if bf16 else g)
    if bf16:
        W0 = to_bf16_f32(W0)
    return W0, grads


@dataclass
class QuadraticProblem:
    """Kronecker-structured quadratic on an m x n matrix parameter."""
    V_L: np.ndarray
    lam_L: np.ndarray
    V_R: np.ndarray
    lam_R: np.ndarray
    W_star: np.ndarray
    W0: np.ndarray
    noise_std: float
    seed: int

    @property
    def H_L(self):
        return (self.V_L * self.lam_L[None, :]) @ self.V_L.T

    @property
    def H_R(self):
        return (self.V_R * self.lam_R[None, :]) @ self.V_R.T

    def gradient(self, W: np.ndarray, t: int) -> np.ndarray:
        """Noisy gradient at W for update step t (noise keyed by (seed, t) so every
        consumer draws the same sample)."""
        noise = np.random.default_rng([self.seed, 7919, int(t)]).standard_normal(self.W0.shape)
        g = self.H_L @ (np.asarray(W, dtype=np.float64) - self.W_star) @ self.H_R
        return (g + self.noise_std * noise).astype(np.float32)

    def loss(self, W: np.ndarray) -> float:
        D = np.asarray(W, dtype=np.float64) - self.W_star
        return 0.5 * float(np.sum(D * (self.H_L @ D @ self.H_R)))


def quadratic_problem(seed: int = 1, m: int = 512, n: int = 128, noise_std: float = 0.01,
                      lam_lo: float = 1e-3, lam_hi: float = 1.0) -> QuadraticProblem:
    rng = np.random.default_rng(seed)
    V_L = haar_orthogonal(rng, m)
    V_R = haar_orthogonal(rng, n)
    lam_L = np.sort(np.exp(rng.uniform(np.log(lam_lo), np.log(lam_hi), m)))[::-1].copy()
    lam_R = np.sort(np.exp(rng.uniform(np.log(lam_lo), np.log(lam_hi), n)))[::-1].copy()
    W_star = rng.standard_normal((m, n))
    W0 = (W_star + rng.standard_normal((m, n))).astype(np.float32)
    return QuadraticProblem(V_L, lam_L, V_R, lam_R, W_star, W0, noise_std, seed)


def fisher_samples(seed: int, V_L, lam_L, V_R, lam_R, count: int):
    """`count` samples G = H_L^{1/2} Z H_R^{1/2} (float64)."""
    rng = np.random.default_rng(seed)
    rootL = (V_L * np.sqrt(lam_L)[None, :]) @ V_L.T
    rootR = (V_R * np.sqrt(lam_R)[None, :]) @ V_R.T
    m, n = V_L.shape[0], V_R.shape[0]
    return [rootL @ rng.standard_normal((m, n)) @ rootR for _ in range(count)]
