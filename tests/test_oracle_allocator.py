"""Pins of the recommendation oracle (oracle/allocator.py): the paper's own worked example (Table 2's underlined
rows), hand-worked traces of Algorithm 1, and brute-force definitions of the Appendix A rules."""
import itertools
import math
import os

import numpy as np
import pytest

from oracle import allocator as oa

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table2_tradeoff.txt")


def table2():
    rows = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        mode, task, layers, acc, speedup, mark = line.split()
        rows.setdefault((mode, task), []).append((int(layers), float(acc), float(speedup), int(mark)))
    return rows


def test_table2_file_is_complete():
    t = table2()
    assert len(t) == 6 and all(len(v) == 7 and [r[0] for r in v] == [0, 2, 4, 6, 8, 10, 12] for v in t.values())
    assert all(sum(r[3] for r in v) == 1 for v in t.values())


@pytest.mark.parametrize("task", ["AFQMC", "IFLYTEK", "TNEWS"])
def test_algorithm_1_reproduces_the_underlined_fully_quant_rows_of_table_2(task):
    """Latency = 1 / speedup.  The three Fully-Quant recommendations (10, 2 and 6 quantised layers) come out of the
    printed listing as it stands."""
    rows = table2()[("fully", task)]
    A = [r[1] for r in rows]
    L = [1.0 / r[2] for r in rows]
    want = [r[0] for r in rows if r[3]][0]
    assert rows[oa.decay_aware_allocate(A, L)][0] == want


def test_algorithm_1_on_the_quant_ffn_only_rows_disagrees_with_the_table():
    """The table is partial (only even layer counts are printed) and the listing, run on the printed rows, picks 2, 8
    and 2 layers where the table underlines 8, 12 and 6.  Recorded so that a change of behaviour is noticed; the
    library follows the listing."""
    got = {}
    for task in ("AFQMC", "IFLYTEK", "TNEWS"):
        rows = table2()[("ffn", task)]
        got[task] = rows[oa.decay_aware_allocate([r[1] for r in rows], [1.0 / r[2] for r in rows])][0]
    assert got == {"AFQMC": 2, "IFLYTEK": 8, "TNEWS": 2}


def test_algorithm_1_hand_traces():
    # one setting: nothing to choose
    assert oa.decay_aware_allocate([0.9], [1.0]) == 0
    # accuracy falls 0.1 per unit of latency gained, then 0.05, then 0.5: rates 0.1, 0.05 (accepted), 0.5 (rejected)
    assert oa.decay_aware_allocate([0.9, 0.8, 0.75, 0.25], [4.0, 3.0, 2.0, 1.0]) == 2
    # a setting that is faster AND more accurate than the recommended one has a negative rate: always accepted,
    # and afterwards positive rates can no longer win (dr_min is negative)
    assert oa.decay_aware_allocate([0.9, 0.95, 0.94], [3.0, 2.0, 1.0]) == 1
    # ... unless they are negative again
    assert oa.decay_aware_allocate([0.9, 0.95, 0.94, 0.96], [4.0, 3.0, 2.0, 1.0]) == 3
    # rates are measured from the last accepted setting, not from FP16: from (0.9, 4) the rates are 0.2 (accepted), then
    # from (0.7, 3): (0.65 - 0.7) / (2 - 3) = 0.05 (accepted); measured from FP16 it would be 0.125 (accepted either way),
    # and the last one (0.3 - 0.65) / (1 - 2) = 0.35 is rejected
    assert oa.decay_aware_allocate([0.9, 0.7, 0.65, 0.3], [4.0, 3.0, 2.0, 1.0]) == 2
    # slower and less accurate: rate (0.8 - 0.9) / (5 - 4) < 0 is accepted by the listing as printed
    assert oa.decay_aware_allocate([0.9, 0.8], [4.0, 5.0]) == 1
    # equal latency: only an accuracy gain is accepted; no change at all is skipped
    assert oa.decay_aware_allocate([0.9, 0.95], [4.0, 4.0]) == 1
    assert oa.decay_aware_allocate([0.9, 0.85], [4.0, 4.0]) == 0
    assert oa.decay_aware_allocate([0.9, 0.9], [4.0, 4.0]) == 0


def test_threshold_rules_against_brute_force():
    rng = np.random.default_rng(5)
    for _ in range(300):
        n = int(rng.integers(1, 9))
        A = np.round(rng.random(n), 2).tolist()
        L = np.round(rng.random(n) + 0.1, 2).tolist()
        thr_l, thr_a = float(np.round(rng.random() + 0.1, 2)), float(np.round(rng.random(), 2))
        got = oa.recommend(A, L, max_latency=thr_l)
        ok = [i for i in range(n) if L[i] <= thr_l]
        if not ok:
            assert got == []
        else:
            assert len(got) == 1 and got[0] in ok and all(A[got[0]] >= A[i] for i in ok)
            assert got[0] == min(i for i in ok if A[i] == A[got[0]])
        got = oa.recommend(A, L, min_accuracy=thr_a)
        ok = [i for i in range(n) if A[i] >= thr_a]
        if not ok:
            assert got == []
        else:
            assert len(got) == 1 and got[0] in ok and all(L[got[0]] <= L[i] for i in ok)
            assert got[0] == min(i for i in ok if L[i] == L[got[0]])


def test_top5_ranking_by_speedup_over_accuracy_loss():
    rows = table2()[("ffn", "IFLYTEK")]
    A = [r[1] for r in rows]
    L = [1.0 / r[2] for r in rows]
    got = oa.recommend(A, L)
    ratio = {i: (L[0] / L[i]) / (A[0] - A[i]) for i in range(1, 7)}
    assert got == sorted(ratio, key=lambda i: -ratio[i])[:5]
    assert got[0] == 1                      # two layers: 1.4 % faster for 0.5 points of accuracy is the best ratio
    # settings that lose no accuracy come first, faster ones first among them
    assert oa.recommend([0.5, 0.5, 0.6, 0.4], [4.0, 3.0, 2.0, 1.0]) == [2, 1, 3]
    assert oa.recommend([0.5], [1.0]) == []
