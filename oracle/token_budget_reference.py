"""TEST INFRASTRUCTURE ONLY -- choosing the token budget from a one-time profile (paper section 4.3,
"Determining Token Budget"; ``compute_token_budget(T_max)`` in the first line of Algorithm 3).

The section fixes the budget by profiling: batches with different numbers of tokens are timed once, and
the budget is the largest number of tokens a batch may hold while an iteration still meets the latency
target T_max (the time-between-tokens objective).  Written out in the plainest form:

    profile : token count -> measured iteration time
    a count tau is SAFE if every profiled count tau' <= tau has  time(tau') <= T_max
    budget  = the largest safe profiled count (none: no budget exists)

Reading, where the section is silent.  Under a budget tau the scheduler builds batches of ANY size up to
tau (Algorithm 3 fills what the running decodes leave), so a budget is only acceptable if the smaller
batches meet the target as well; for a profile that grows with the token count, which the section takes
for granted, this is the same as "the largest count whose own time meets the target".  "Meets" is
``<=``: a batch that takes exactly T_max is within the objective.

No arithmetic is shared with the product (``paper_2403_02310_amd/token_budget.py``), which this checks.
"""
from __future__ import annotations

from typing import Dict, Optional


def compute_token_budget(profile: Dict[int, float], t_max: float) -> Optional[int]:
    """``profile`` maps a profiled token count to its measured iteration time (same unit as ``t_max``)."""
    best = None
    for tau in profile:                       # every candidate, in no particular order
        safe = True
        for other, seconds in profile.items():
            if other <= tau and not (seconds <= t_max):
                safe = False
        if safe and (best is None or tau > best):
            best = tau
    return best
