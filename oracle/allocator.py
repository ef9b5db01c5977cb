"""Oracle of the mixed-precision recommendation logic (plain Python, binary64).

TEST INFRASTRUCTURE ONLY, like the rest of this package.

Two procedures of the paper, written in its notation:

* decay_aware_allocate(A, L): the Accuracy-Decay-Aware allocator (Section 3.2, Algorithm 1).  A[i], L[i] are the
  accuracy and the latency of setting i of a mode (i = 0 is the all-FP16 setting, larger i quantises more layers);
  the result Lq is the index of the recommended setting.
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


def decay_aware_allocate(A: Sequence[float], L: Sequence[float]) -> int:
    """Algorithm 1.  Walks the settings in order, keeping a recommended setting (A_rec, L_rec); setting i replaces it
    when its decay rate dr = (A_i - A_rec) / (L_i - L_rec) is negative or smaller than the smallest rate seen."""
    assert len(A) == len(L) and len(A) >= 1
    dr_min = math.inf                       # MAX_FLOAT
    A_rec, L_rec, Lq = A[0], L[0], 0        # i == 0: the FP16 setting
    for i in range(1, len(A)):
        dA, dL = A[i] - A_rec, L[i] - L_rec
        if dL == 0.0:
            if dA == 0.0:
                continue
            dr = -math.inf if dA > 0.0 else math.inf
        else:
            dr = dA / dL
        if dr < 0.0 or dr < dr_min:
            dr_min = dr
            A_rec, L_rec, Lq = A[i], L[i], i
    return Lq


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
