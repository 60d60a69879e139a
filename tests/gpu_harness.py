"""Side-by-side driver for the parity tests: the same seeded inputs go to the CPU
oracle (float64) and, through the C ABI, to the HIP library."""
from __future__ import annotations

import numpy as np
import torch

from oracle import br_oracle as oc
from oracle.metrics import orthogonality_defect, rel_err  # noqa: F401  (re-exported for the tests)


def f32(x):
    return float(np.float32(x))


def oracle_hyper(**kw):
    geometry = {0: "bilateral", 1: "unilateral"}[kw.pop("geometry", 0)]
    source = {0: "second", 1: "first"}[kw.pop("source", 0)]
    sb = kw.pop("stat_beta", -1.0)
    hp = oc.Hyper(beta1=kw.pop("beta1", 0.9), beta2=kw.pop("beta2", 0.95), eps=kw.pop("eps", 1e-8),
                  weight_decay=kw.pop("weight_decay", 0.0), stat_beta=None if sb < 0 else sb,
                  geometry=geometry, source=source, power_iters=kw.pop("power_iters", 1),
                  bias_correction=bool(kw.pop("bias_correction", 0)),
                  eps_outside_sqrt=bool(kw.pop("eps_outside_sqrt", 0)),
                  stats_on_refresh_only=bool(kw.pop("stats_on_refresh_only", 0)))
    kw.pop("compute_norms", None)
    kw.pop("math", None)
    kw.pop("cache_rotated_moment", None)
    kw.pop("refresh_math", None)
    assert not kw, kw
    return hp.rounded_to_f32()


def to_dev(a, bf16=False):
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).cuda()
    return t.to(torch.bfloat16).contiguous() if bf16 else t


def to_np(t):
    return t.detach().to(torch.float32).cpu().numpy().astype(np.float64)


class SideBySide:
    """Runs a list of matrices through both implementations, step by step."""

    def __init__(self, W0s, freq, lr, rotate=None, bf16_params=False, bf16_grads=False, qr=None, **hparams):
        from paper_2602_03515_amd import binding as B
        from paper_2602_03515_amd.optimizer import BasisRotationAdam
        self.B = B
        self.freq, self.lr = freq, f32(lr)
        self.bf16_params, self.bf16_grads = bf16_params, bf16_grads
        self.hp = oracle_hyper(**dict(hparams))
        self.qr = qr or oc.householder_qr
        rot = [True] * len(W0s) if rotate is None else rotate
        self.states = [oc.MatrixState(W.shape[0], W.shape[1], self.hp, r) for W, r in zip(W0s, rot)]
        self.W_ref = [np.asarray(W, dtype=np.float64).copy() for W in W0s]
        self.params = [to_dev(W, bf16_params) for W in W0s]
        self.opt = BasisRotationAdam(self.params, freq=freq, lr=self.lr, rotate=rot,
                                     grad_dtype=torch.bfloat16 if bf16_grads else torch.float32, **hparams)

    def step(self, grads, lr=None):
        lr = self.lr if lr is None else f32(lr)
        g_dev = [to_dev(g, self.bf16_grads) for g in grads]
        self.opt.step(g_dev, lr)
        torch.cuda.synchronize()
        for i, (st, g) in enumerate(zip(self.states, grads)):
            self.W_ref[i] = oc.optimizer_step(st, self.W_ref[i], np.asarray(g, dtype=np.float64), lr, self.hp,
                                              self.freq, self.qr)

    def gpu_weights(self, i):
        if self.bf16_params and self.opt.step_count > 0:    # the master copy exists from the first step on
            return to_np(self.opt.state(i, self.B.BR_STATE_MASTER))
        return to_np(self.params[i])

    def compare_state(self, tol, q_tol=None, check_q=True):
        B = self.B
        worst = {}
        for i, st in enumerate(self.states):
            pairs = [("W", self.gpu_weights(i), self.W_ref[i]),
                     ("M", to_np(self.opt.state(i, B.BR_STATE_M)), st.M),
                     ("S", to_np(self.opt.state(i, B.BR_STATE_S)), st.S)]
            if st.L is not None:
                pairs.append(("L", to_np(self.opt.state(i, B.BR_STATE_L)), st.L))
            if st.R is not None:
                pairs.append(("R", to_np(self.opt.state(i, B.BR_STATE_R)), st.R))
            if check_q and st.QL is not None:
                pairs.append(("QL", to_np(self.opt.state(i, B.BR_STATE_QL)), st.QL))
            if check_q and st.QR is not None:
                pairs.append(("QR", to_np(self.opt.state(i, B.BR_STATE_QR)), st.QR))
            for name, a, b in pairs:
                e = rel_err(a, b)
                worst[name] = max(worst.get(name, 0.0), e)
                lim = (q_tol if (q_tol is not None and name in ("QL", "QR")) else tol)
                assert e <= lim, f"matrix {i} {name}: rel err {e:.3e} > {lim:.1e}"
        return worst
