"""Host-side ring of delayed gradients (the hand-off in front of the optimizer step).

Under a delay of tau updates the gradient applied at update step t was evaluated at
the iterate W_{max(t-1-tau, 0)} (Appendix B, the delayed-gradient equation).  In an
asynchronous pipeline the backward pass of a stage produces such gradients on its
own; this helper reproduces the indexing for synthetic drivers.  It only moves
references: no copy, no arithmetic.
"""
from __future__ import annotations

from collections import deque


def delayed_index(t: int, tau: int) -> int:
    """Index s of the iterate W_s whose gradient update step t (1-based) consumes."""
    if t < 1 or tau < 0:
        raise ValueError("t starts at 1 and tau is non-negative")
    return 0 if t <= tau else t - 1 - tau


class GradientRing:
    """Keeps the last tau+1 pushed items (weight snapshots or gradient buffers).

    Usage with weight snapshots: push W_0 once, then at every step t call
    `stale()` to get W_{max(t-1-tau,0)}, evaluate the gradient there, update, and
    push the new iterate W_t.
    """

    def __init__(self, tau: int):
        if tau < 0:
            raise ValueError("tau must be non-negative")
        self.tau = int(tau)
        self._slots = deque(maxlen=self.tau + 1)

    def push(self, item) -> None:
        self._slots.append(item)

    def stale(self):
        """Oldest retained item: W_{t-1-tau} once tau+1 items exist, W_0 before."""
        if not self._slots:
            raise IndexError("ring is empty")
        return self._slots[0]

    def __len__(self) -> int:
        return len(self._slots)
