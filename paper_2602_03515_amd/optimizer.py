"""Thin torch-facing driver over the C ABI: owns the workspace tensor, builds the
pointer arrays and applies the refresh schedule `t mod freq == 0` of Algorithm 1.
All arithmetic happens inside the HIP library."""
from __future__ import annotations

from typing import Optional, Sequence

import torch

from . import binding as B

_DT = {torch.float32: B.BR_F32, torch.bfloat16: B.BR_BF16}


class BasisRotationAdam:
    def __init__(self, params: Sequence[torch.Tensor], freq: int = 10, lr: float = 1e-3,
                 rotate: Optional[Sequence[bool]] = None, grad_dtype: Optional[torch.dtype] = None, **hparams):
        if not params:
            raise ValueError("no parameters")
        dev = params[0].device
        if dev.type != "cuda":
            raise RuntimeError("BasisRotationAdam runs on the GPU only; there is no CPU path")
        for p in params:
            if p.dim() != 2 or not p.is_contiguous() or p.device != dev or p.dtype not in _DT:
                raise ValueError("parameters must be contiguous 2-D float32/bfloat16 tensors on one GPU")
        self.params = list(params)
        self.freq = int(freq)
        self.lr = float(lr)
        rot = [True] * len(params) if rotate is None else [bool(r) for r in rotate]
        shapes = [(p.shape[0], p.shape[1], _DT[p.dtype], _DT[grad_dtype or p.dtype], int(r))
                  for p, r in zip(self.params, rot)]
        self.descs = B.make_descs(shapes)
        self.hp = B.make_hparams(**hparams)
        self.state_bytes, self.scratch_bytes = B.br_workspace_bytes(self.descs, self.hp)
        self.workspace = torch.empty(self.state_bytes + self.scratch_bytes, dtype=torch.uint8, device=dev)
        self.stream = torch.cuda.current_stream(dev)
        self.ctx = B.br_init(self.descs, self.hp, self.workspace.data_ptr(), self.workspace.numel(),
                             self.stream.cuda_stream)

    # -- the three calls of one optimizer step, in Algorithm 1's order ---------------------
    def accumulate_stats(self, grads: Sequence[torch.Tensor]) -> None:
        self._check_grads(grads)
        B.br_accumulate_stats(self.ctx, [g.data_ptr() for g in grads])

    def delay_compensate(self, grads: Sequence[torch.Tensor], stale_params: Sequence[torch.Tensor], lam: float) -> None:
        """G <- G + lam G.G.(W - W_stale) in place, W the current parameters."""
        B.br_delay_compensate(self.ctx, [g.data_ptr() for g in grads], [p.data_ptr() for p in self.params],
                              [p.data_ptr() for p in stale_params], float(lam))

    def clip_gradients(self, grads: Sequence[torch.Tensor], max_norm: float) -> None:
        """Global-norm clipping of the stage's gradients, in place, on the device."""
        self._check_grads(grads)
        B.br_clip_gradients(self.ctx, [g.data_ptr() for g in grads], float(max_norm))

    def clip_result(self) -> torch.Tensor:
        """Device tensor [global norm, applied factor] of the latest clip_gradients call."""
        off = B.br_get_clip_result(self.ctx) - self.workspace.data_ptr()
        return self.workspace[off:off + 8].view(torch.float32)

    def refresh_basis(self) -> None:
        B.br_refresh_basis(self.ctx)

    def apply(self, grads: Sequence[torch.Tensor], lr: Optional[float] = None) -> None:
        self._check_grads(grads)
        B.br_step(self.ctx, [p.data_ptr() for p in self.params], [g.data_ptr() for g in grads],
                  self.lr if lr is None else float(lr))

    def step(self, grads: Sequence[torch.Tensor], lr: Optional[float] = None,
             max_grad_norm: Optional[float] = None) -> None:
        t = self.step_count + 1
        if max_grad_norm is not None:
            self.clip_gradients(grads, max_grad_norm)
        self.accumulate_stats(grads)
        if self.freq > 0 and t % self.freq == 0:
            self.refresh_basis()
        self.apply(grads, lr)

    # -- state access ----------------------------------------------------------------------
    @property
    def step_count(self) -> int:
        return B.br_get_step_count(self.ctx)

    def state(self, mat: int, which: int) -> torch.Tensor:
        """Zero-copy float32 view of one state buffer inside the workspace."""
        ptr, rows, cols = B.br_get_state(self.ctx, mat, which)
        off = ptr - self.workspace.data_ptr()
        return self.workspace[off:off + rows * cols * 4].view(torch.float32).view(rows, cols)

    def has_state(self, mat: int, which: int) -> bool:
        try:
            B.br_get_state(self.ctx, mat, which)
            return True
        except B.BrError:
            return False

    def _check_grads(self, grads):
        if len(grads) != len(self.params):
            raise ValueError("one gradient per parameter")
        for i, (g, p) in enumerate(zip(grads, self.params)):
            want = B.BR_BF16 if self.descs[i].grad_dtype == B.BR_BF16 else B.BR_F32
            if g.shape != p.shape or not g.is_contiguous() or g.device != p.device or _DT.get(g.dtype) != want:
                raise ValueError(f"gradient {i} does not match its descriptor")

    def close(self) -> None:
        if getattr(self, "ctx", None):
            B.br_destroy(self.ctx)
            self.ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
