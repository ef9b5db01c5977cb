"""Parity of the library's recommendation functions (samp_allocate_decay_aware, samp_recommend) with the oracle.
They are host functions of the C-ABI library and launch nothing, so the parity cases run without a GPU; the last
test feeds them latencies measured on the GPU."""
import math
import os

import numpy as np
import pytest

from oracle import allocator as oa

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "table2_tradeoff.txt")


@pytest.fixture(scope="module")
def P():
    import paper_2209_09130_amd as P
    from paper_2209_09130_amd import build as B
    if not os.path.exists(P.lib_path()):
        B.build(force=True)
    P.lib()
    return P


def curves():
    rows = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        mode, task, layers, acc, speedup, mark = line.split()
        rows.setdefault((mode, task), []).append((float(acc), 1.0 / float(speedup)))
    return {k: ([a for a, _ in v], [l for _, l in v]) for k, v in rows.items()}


def random_curves(rng):
    n = int(rng.integers(1, 14))
    kind = int(rng.integers(0, 3))
    if kind == 0:                                        # coarse grid: many exact ties and equal latencies
        return np.round(rng.random(n), 1).tolist(), (np.round(rng.random(n), 1) + 0.5).tolist()
    if kind == 1:                                        # the usual shape: latency falls, accuracy decays with noise
        L = np.sort(rng.random(n) + 0.2)[::-1].tolist()
        A = (0.9 - np.cumsum(rng.random(n) * 0.05) + rng.standard_normal(n) * 0.01).tolist()
        return A, L
    return rng.random(n).tolist(), (rng.random(n) + 0.1).tolist()


def test_table2_curves(P):
    for key, (A, L) in curves().items():
        assert P.allocate_decay_aware(A, L) == oa.decay_aware_allocate(A, L), key
        assert P.recommend(A, L) == oa.recommend(A, L), key
        for thr in (L[0], L[3], L[-1], L[-1] * 0.5):
            assert P.recommend(A, L, max_latency=thr) == oa.recommend(A, L, max_latency=thr), key
        for thr in (A[0], 0.5, 0.0, 1.0):
            assert P.recommend(A, L, min_accuracy=thr) == oa.recommend(A, L, min_accuracy=thr), key


def test_random_curves_including_ties_and_single_settings(P):
    rng = np.random.default_rng(11)
    for _ in range(2000):
        A, L = random_curves(rng)
        assert P.allocate_decay_aware(A, L) == oa.decay_aware_allocate(A, L), (A, L)
        assert P.recommend(A, L) == oa.recommend(A, L), (A, L)
        tl, ta = float(rng.choice(L)) if rng.random() < 0.5 else float(rng.random() + 0.3), float(rng.choice(A))
        assert P.recommend(A, L, max_latency=tl) == oa.recommend(A, L, max_latency=tl), (A, L, tl)
        assert P.recommend(A, L, min_accuracy=ta) == oa.recommend(A, L, min_accuracy=ta), (A, L, ta)


def test_argument_errors(P):
    with pytest.raises(P.SampError):
        P.allocate_decay_aware([], [])
    with pytest.raises(P.SampError):
        P.allocate_decay_aware([0.5, float("nan")], [1.0, 0.5])
    with pytest.raises(P.SampError):
        P.allocate_decay_aware([0.5, 0.4], [1.0, 0.0])
    with pytest.raises(P.SampError):
        P.allocate_decay_aware([0.5] * 65, [1.0] * 65)
    with pytest.raises(P.SampError):
        P.recommend([0.5, 0.4], [1.0, 0.5], max_latency=math.inf)


@pytest.mark.gpu
def test_recommendation_from_latencies_measured_on_the_gpu(P):
    """Quant-FFN-Only settings 0, 2, .., 12 of a 12-layer encoder (first layers quantised, as in Table 2's layer counts):
    latencies measured with the library, accuracies taken from the table's AFQMC column (no dataset here)."""
    import torch
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import samp_workloads as W
    from paper_2209_09130_amd import tradeoff
    w = W.config("C2")
    lat = tradeoff.measure_latencies(w, mode=W.FFN_INT8, counts=range(0, 13, 2), steps=20, warmup=5)
    assert len(lat) == 7 and all(v > 0 for v in lat)
    assert lat[-1] < lat[0]                                # twelve quantised FFN blocks are faster than none
    A = curves()[("ffn", "AFQMC")][0]
    assert P.allocate_decay_aware(A, lat) == oa.decay_aware_allocate(A, lat)
    assert P.recommend(A, lat, max_latency=lat[3]) == oa.recommend(A, lat, max_latency=lat[3])
