"""Host-side refresh schedules.  The library refreshes whenever `br_refresh_basis` is called;
when to call it is policy.  Uniform: every `freq` steps (Algorithm 1).  Stage-aware: the paper
allocates the refresh budget of a pipeline stage in proportion to its gradient delay at equal
total cost (Section 4.3, "Stage-aware" paragraph; the closed-form rule printed in the appendix
divides by zero for a delay of one step and is not used)."""
from __future__ import annotations

from typing import List, Sequence


def stage_refresh_periods(delays: Sequence[float], base_period: int) -> List[int]:
    """Refresh period (in steps) for every stage.  `delays[k]` is the gradient delay tau of
    stage k.  Budgets 1/period are proportional to the delays and sum to
    len(delays) / base_period; a stage without delay never refreshes (period 0).  Periods are
    rounded to the nearest step, at least 1."""
    if base_period < 1:
        raise ValueError("base_period must be at least 1")
    total = float(sum(delays))
    if any(d < 0 for d in delays):
        raise ValueError("delays are non-negative")
    if total <= 0:
        return [int(base_period)] * len(delays)
    budget = len(delays) / float(base_period)
    return [0 if d <= 0 else max(1, int(round(total / (budget * d)))) for d in delays]


def refresh_due(t: int, period: int) -> bool:
    """True when update step t (1-based) refreshes under `period` (0 = never)."""
    return period > 0 and t % period == 0
