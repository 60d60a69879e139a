"""Float64 CPU oracle of the basis-rotation Adam step (TEST INFRASTRUCTURE ONLY).

What is restated here, and where the paper defines it:

  * first moment kept in the ORIGINAL space            -- Algorithm 1, first-moment update;
    Appendix "Connection to Recent Optimizers" (momentum accumulated in
    the original space, basis refreshed before the optimisation step)
  * Kronecker-factor statistics L, R as EMAs of G G^T, G^T G
                                                       -- Algorithm 2, updates of L and R
  * Power(A, Q): one multiplication by A followed by a QR factorisation,
    Q <- qr(A Q).Q                                     -- Section 3.2, last paragraph
  * unilateral geometry rotates only the smaller side  -- Algorithm 2, unilateral branch
    together with Section 3.2 / the memory-overhead appendix (min(m, n)^2)
  * rotate, second moment in the rotated basis, rotate back
                                                       -- Algorithm 1, rotation to update
  * epsilon INSIDE the square root, no bias correction -- Algorithm 1, update formula
    and the "standard Adam update" equation of Section 3.1
  * delayed-gradient indexing                          -- Appendix B, the
    delayed-gradient case equation

Readings taken where the paper is silent (each is a keyword argument so the
other reading can be run):
  * statistics are accumulated every step (the refresh itself stays on the
    paper's `t mod freq == 0` schedule);
  * U, V start as identity matrices;
  * `power_iters` multiplications are followed by ONE QR;
  * QR is made unique by requiring diag(R) >= 0 (a zero counts as +);
  * no re-sorting of columns and no re-rotation of the second moment when
    the basis changes;
  * decoupled weight decay  W <- W - lr*wd*W  is applied to the pre-step W;
  * bf16 parameters are the round-to-nearest-even image of a full-precision
    master copy that receives the update.

All arithmetic is float64.  Nothing here is blocked, fused or reordered.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Callable, Optional

import numpy as np

__all__ = [
    "Hyper", "MatrixState", "rotated_sides", "householder_qr", "power_qr",
    "ingest", "refresh", "step", "optimizer_step", "bf16_round",
    "delayed_weight_index", "run_fixed_gradients", "run_delayed",
]


@dataclass
class Hyper:
    """Hyper-parameters of Algorithm 1/2.  Values are used as given; callers
    comparing against a float32 ABI pass float32-rounded numbers."""
    beta1: float = 0.9
    beta2: float = 0.95
    eps: float = 1e-8
    weight_decay: float = 0.0
    stat_beta: Optional[float] = None      # None -> beta2 (Algorithm 2, update of L)
    geometry: str = "bilateral"            # "bilateral" | "unilateral"
    source: str = "second"                 # "second" (L, R buffers) | "first" (M M^T, M^T M)
    power_iters: int = 1
    bias_correction: bool = False          # textbook-Adam option, not in Algorithm 1
    eps_outside_sqrt: bool = False         # textbook-Adam option, not in Algorithm 1
    stats_on_refresh_only: bool = False    # literal reading of Algorithm 2 inside Algorithm 1

    def rounded_to_f32(self) -> "Hyper":
        f = lambda x: float(np.float32(x))
        return Hyper(f(self.beta1), f(self.beta2), f(self.eps), f(self.weight_decay),
                     None if self.stat_beta is None else f(self.stat_beta),
                     self.geometry, self.source, self.power_iters,
                     self.bias_correction, self.eps_outside_sqrt,
                     self.stats_on_refresh_only)


def rotated_sides(m: int, n: int, geometry: str, rotate: bool = True):
    """Which sides carry a rotation.  Bilateral: both.  Unilateral: the side of
    size min(m, n); a square matrix keeps the left factor as Algorithm 2 does."""
    if not rotate:
        return False, False
    if geometry == "bilateral":
        return True, True
    if geometry == "unilateral":
        return (True, False) if m <= n else (False, True)
    raise ValueError(f"unknown geometry {geometry!r}")


class MatrixState:
    """Optimizer state of one m x n weight matrix (memory-overhead appendix):
    M, S (m x n), L, Q_L (m x m), R, Q_R (n x n); absent factors are None."""

    def __init__(self, m: int, n: int, hp: Hyper, rotate: bool = True):
        self.m, self.n = int(m), int(n)
        self.rot_left, self.rot_right = rotated_sides(m, n, hp.geometry, rotate)
        self.M = np.zeros((m, n))
        self.S = np.zeros((m, n))
        keep_stats = hp.source == "second"
        self.L = np.zeros((m, m)) if (self.rot_left and keep_stats) else None
        self.R = np.zeros((n, n)) if (self.rot_right and keep_stats) else None
        self.QL = np.eye(m) if self.rot_left else None
        self.QR = np.eye(n) if self.rot_right else None
        self.t = 0                     # completed optimizer steps
        self.last = {}                 # intermediates of the latest step (for tests)


def householder_qr(P: np.ndarray):
    """QR factorisation by Householder reflections, made unique by diag(R) >= 0.

    Returns (Q, R) with Q square orthogonal, R upper triangular, Q @ R == P.
    Column j is reduced by H_j = I - 2 v v^T / (v^T v), v = x + sign(x_0)|x| e_0,
    the textbook choice that avoids cancellation.  A zero column is skipped.
    """
    A = np.array(P, dtype=np.float64, copy=True)
    rows, cols = A.shape
    Q = np.eye(rows)
    for j in range(min(rows, cols)):
        x = A[j:, j]
        normx = np.sqrt(x @ x)
        if normx == 0.0:
            continue
        v = x.copy()
        v[0] += np.copysign(normx, x[0])
        vv = v @ v
        A[j:, j:] -= np.outer(v, (2.0 / vv) * (v @ A[j:, j:]))
        Q[:, j:] -= np.outer(Q[:, j:] @ v, (2.0 / vv) * v)
    R = np.triu(A)
    d = np.where(np.diag(R) < 0.0, -1.0, 1.0)
    k = d.shape[0]
    Q[:, :k] *= d[None, :]
    R[:k, :] *= d[:, None]
    return Q, R


def power_qr(A: np.ndarray, Q: np.ndarray, iters: int = 1,
             qr: Callable = householder_qr) -> np.ndarray:
    """Power(A, Q): multiply `iters` times by A, then orthonormalise once."""
    P = np.array(Q, dtype=np.float64, copy=True)
    for _ in range(int(iters)):
        P = A @ P
    return qr(P)[0]


def ingest(st: MatrixState, G: np.ndarray, hp: Hyper, update_stats: bool = True) -> None:
    """Consume the step's (delayed) gradient: first moment and, for the
    second-order source, the Kronecker-factor statistics."""
    G = np.asarray(G, dtype=np.float64)
    st.M = hp.beta1 * st.M + (1.0 - hp.beta1) * G
    if hp.source == "second" and update_stats:
        b = hp.beta2 if hp.stat_beta is None else hp.stat_beta
        if st.L is not None:
            st.L = b * st.L + (1.0 - b) * (G @ G.T)
        if st.R is not None:
            st.R = b * st.R + (1.0 - b) * (G.T @ G)


def refresh(st: MatrixState, hp: Hyper, qr: Callable = householder_qr) -> None:
    """Eigenbasis-Estimation for every rotated side of one matrix."""
    if st.rot_left:
        A = st.L if hp.source == "second" else st.M @ st.M.T
        st.QL = power_qr(A, st.QL, hp.power_iters, qr)
    if st.rot_right:
        A = st.R if hp.source == "second" else st.M.T @ st.M
        st.QR = power_qr(A, st.QR, hp.power_iters, qr)


def step(st: MatrixState, W: np.ndarray, G: np.ndarray, lr: float, hp: Hyper) -> np.ndarray:
    """Algorithm 1 from the rotation of G and M to the parameter update, for one matrix; returns the new weights.
    `st.M` must already contain this step's gradient (see `ingest`)."""
    W = np.asarray(W, dtype=np.float64)
    G = np.asarray(G, dtype=np.float64)
    st.t += 1
    Gt, Mt = G, st.M
    if st.rot_left:
        Gt = st.QL.T @ Gt
        Mt = st.QL.T @ Mt
    if st.rot_right:
        Gt = Gt @ st.QR
        Mt = Mt @ st.QR
    st.S = hp.beta2 * st.S + (1.0 - hp.beta2) * (Gt * Gt)
    num, den = Mt, st.S
    if hp.bias_correction:
        num = Mt / (1.0 - hp.beta1 ** st.t)
        den = st.S / (1.0 - hp.beta2 ** st.t)
    if hp.eps_outside_sqrt:
        X = num / (np.sqrt(den) + hp.eps)
    else:
        X = num / np.sqrt(den + hp.eps)
    dW = X
    if st.rot_left:
        dW = st.QL @ dW
    if st.rot_right:
        dW = dW @ st.QR.T
    st.last = {"G_rot": Gt, "M_rot": Mt, "X": X, "dW": dW}
    return W - lr * dW - lr * hp.weight_decay * W


def optimizer_step(st: MatrixState, W: np.ndarray, G: np.ndarray, lr: float, hp: Hyper,
                   freq: int, qr: Callable = householder_qr) -> np.ndarray:
    """One iteration of Algorithm 1 in the paper's order: first moment (and
    statistics), refresh when t mod freq == 0, rotated Adam update."""
    t = st.t + 1
    do_refresh = freq > 0 and (t % freq == 0)
    ingest(st, G, hp, update_stats=(not hp.stats_on_refresh_only) or do_refresh)
    if do_refresh and (st.rot_left or st.rot_right):
        refresh(st, hp, qr)
    return step(st, W, G, lr, hp)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """Round to the nearest bfloat16 (ties to even), returned as float64.
    The value passes through float32 first; bfloat16 keeps the top 16 bits."""
    f = np.ascontiguousarray(np.asarray(x, dtype=np.float64).astype(np.float32))
    bits = f.view(np.uint32).astype(np.uint64)
    lsb = (bits >> np.uint64(16)) & np.uint64(1)
    rounded = (bits + np.uint64(0x7FFF) + lsb) & np.uint64(0xFFFF0000)
    out = rounded.astype(np.uint32).view(np.float32).astype(np.float64)
    nan = np.isnan(f)
    if nan.any():
        out = np.where(nan, np.nan, out)
    return out.reshape(np.shape(x))


def delayed_weight_index(t: int, tau: int) -> int:
    """Index s of the iterate W_s at which the gradient consumed by update
    step t (1-based) was evaluated under a delay of tau updates."""
    return 0 if t <= tau else t - 1 - tau


def run_fixed_gradients(W0, grads, hp: Hyper, lr, freq: int, rotate: bool = True,
                        qr: Callable = householder_qr, bf16_params: bool = False):
    """Run Algorithm 1 on a pre-generated gradient sequence (gradients that do
    not depend on the weights, so a delay only renames buffers).  Returns the
    state and the list of weights after each step (and the bf16 images)."""
    W0 = np.asarray(W0, dtype=np.float64)
    st = MatrixState(W0.shape[0], W0.shape[1], hp, rotate)
    W = W0.copy()
    history = []
    for i, G in enumerate(grads):
        eta = lr[i] if np.ndim(lr) else lr
        W = optimizer_step(st, W, G, eta, hp, freq, qr)
        history.append(bf16_round(W) if bf16_params else W.copy())
    return st, W, history


def run_delayed(grad_fn: Callable, W0, hp: Hyper, lr: float, freq: int, tau: int, steps: int,
                rotate: bool = True, qr: Callable = householder_qr, record=None):
    """Run Algorithm 1 with weight-dependent gradients under a delay of `tau`
    updates: update step t consumes grad_fn(W_s, t) with s given by
    `delayed_weight_index`.  Returns (state, final W, list of consumed gradients)."""
    W0 = np.asarray(W0, dtype=np.float64)
    st = MatrixState(W0.shape[0], W0.shape[1], hp, rotate)
    iterates = [W0.copy()]
    consumed = []
    for t in range(1, steps + 1):
        G = np.asarray(grad_fn(iterates[delayed_weight_index(t, tau)], t), dtype=np.float64)
        consumed.append(G)
        W = optimizer_step(st, iterates[-1], G, lr, hp, freq, qr)
        iterates.append(W)
        if len(iterates) > tau + 2:          # only the last tau+1 iterates are ever read
            iterates[-(tau + 3)] = None
        if record is not None:
            record(t, st, W)
    return st, iterates[-1], consumed


def extra_state_floats(m: int, n: int, geometry: str, source: str) -> int:
    """Floats of state beyond Adam's two moments (memory-overhead appendix, table):
    rotation matrices, plus the statistics buffers for the second-order source."""
    left, right = rotated_sides(m, n, geometry)
    rot = (m * m if left else 0) + (n * n if right else 0)
    return rot * (2 if source == "second" else 1)


def clip_by_global_norm(grads, max_norm: float):
    """Global-norm gradient clipping as used in the paper's training recipe (experimental details:
    clipping value 1.0): every gradient is multiplied by min(1, max_norm / (norm + 1e-6)) with
    norm the 2-norm of all entries of all gradients.  Returns (scaled gradients, norm, factor)."""
    total = 0.0
    for g in grads:
        g64 = np.asarray(g, dtype=np.float64)
        total += float(np.sum(g64 * g64))
    norm = float(np.sqrt(total))
    factor = min(1.0, max_norm / (norm + 1e-6))
    return [np.asarray(g, dtype=np.float64) * factor for g in grads], norm, factor


def delay_compensate(G, W_now, W_stale, lam: float):
    """Delay Compensation (appendix "Experiments for Other Baselines", the displayed first-order
    Taylor formula): the gradient taken at the stale weights is corrected towards the current
    weights with the diagonal empirical Fisher as the Hessian,
        g <- g + lam * g . g . (w_now - w_stale),     lam in [0, 1]."""
    g = np.asarray(G, dtype=np.float64)
    return g + lam * g * g * (np.asarray(W_now, dtype=np.float64) - np.asarray(W_stale, dtype=np.float64))


def stage_refresh_periods(delays, base_period: int):
    """Stage-aware refresh allocation (Section 4.3, "Stage-aware" paragraph): the refresh budget
    of a stage, 1 / period, is proportional to its gradient delay, and the total budget equals
    that of a uniform schedule with `base_period` on every stage.  A stage without delay gets no
    refreshes (period 0 = never).  Periods are real numbers here; callers round."""
    delays = [float(d) for d in delays]
    total = sum(delays)
    if total <= 0:
        return [float(base_period)] * len(delays)
    budget = len(delays) / float(base_period)
    return [0.0 if d <= 0 else total / (budget * d) for d in delays]
