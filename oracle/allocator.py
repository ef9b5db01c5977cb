"""Oracle of the mixed-precision recommendation logic (plain Python, binary64).

TEST INFRASTRUCTURE ONLY, like the rest of this package.

Two procedures of the paper:

* decay_aware_allocate(A, L): the Accuracy-Decay-Aware allocator (Section 3.2, Algorithm 1).  A[i], L[i] are the
  accuracy and the latency of setting i of a mode (i = 0 is the all-FP16 setting, larger i quantises more layers);
  the result is the index of the recommended setting.
* recommend(A, L, max_latency, min_accuracy): the threshold rules of Appendix A.

Readings where the paper is silent (the library takes the same readings):
* L is a latency (time per inference).  Table 2 prints speedups; its rows are turned into latencies as 1/speedup.
* L[i] == L_rec makes the decay rate a division by zero: the rate is taken as -inf if the accuracy rose (accepted,
  like any negative rate), +inf if it fell (never accepted), and the setting is skipped if both are unchanged.
* Appendix A's "lower than" / "higher than" thresholds are inclusive; ties go to the setting with fewer quantised
  layers; with neither threshold the ranking is by (L[0]/L[i]) / (A[0] - A[i]) over i >= 1, a setting that loses no
  accuracy ranking above all that do (among those by speedup), at most five settings returned.
"""
from __future__ import annotations

import math
from typing import List, Optional, Sequence


def decay_rate(A: Sequence[float], L: Sequence[float], frm: int, to: int) -> Optional[float]:
    """Accuracy change per unit of latency change when moving from setting `frm` to setting `to`.  Equal latencies
    (the quotient is undefined): -inf for an accuracy gain, +inf for a loss, None when nothing changes."""
    gain, cost = A[to] - A[frm], L[to] - L[frm]
    if cost != 0.0:
        return gain / cost
    if gain == 0.0:
        return None
    return -math.inf if gain > 0.0 else math.inf


def decay_aware_allocate(A: Sequence[float], L: Sequence[float]) -> int:
    """Algorithm 1.  One pass over the settings in order of increasing quantisation, starting from the all-FP16
    setting.  A candidate takes over as the recommendation when its decay rate against the current recommendation is
    negative, or lower than every rate that has taken over before; the rate it took over with becomes the bar for
    the candidates after it."""
    assert len(A) == len(L) and len(A) >= 1
    chosen, bar = 0, math.inf
    for cand in range(1, len(A)):
        rate = decay_rate(A, L, chosen, cand)
        if rate is not None and (rate < 0.0 or rate < bar):
            chosen, bar = cand, rate
    return chosen


def recommend(A: Sequence[float], L: Sequence[float], max_latency: Optional[float] = None,
              min_accuracy: Optional[float] = None) -> List[int]:
    """Appendix A.  With a latency threshold: the most accurate setting whose latency does not exceed it.  Else with
    an accuracy threshold: the fastest setting whose accuracy is not below it.  Else: up to five settings ranked by
    speedup over accuracy loss.  Returns setting indices, best first ([] if no setting qualifies)."""
    n = len(A)
    assert n == len(L) and n >= 1
    if max_latency is not None:
        ok = [i for i in range(n) if L[i] <= max_latency]
        if not ok:
            return []
        best = ok[0]
        for i in ok[1:]:
            if A[i] > A[best]:
                best = i
        return [best]
    if min_accuracy is not None:
        ok = [i for i in range(n) if A[i] >= min_accuracy]
        if not ok:
            return []
        best = ok[0]
        for i in ok[1:]:
            if L[i] < L[best]:
                best = i
        return [best]
    keyed = []
    for i in range(1, n):
        speedup = L[0] / L[i]
        loss = A[0] - A[i]
        lossless = loss <= 0.0
        ratio = math.inf if lossless else speedup / loss
        keyed.append((0 if lossless else 1, -ratio if not lossless else -speedup, i))
    keyed.sort()
    return [i for _, _, i in keyed[:5]]
