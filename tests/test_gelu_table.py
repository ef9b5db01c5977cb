"""The FFN1 epilogue's threshold table (a host function of the library) against the oracle's definition
code = rne(GELU(y) / s_out): no GPU needed.  The lookup is emulated here with the documented bin map
(one binary32 fused multiply-add, a clamp, the low mantissa bits) and must return the oracle's code for
every y tried: dense sweeps, random values, and the binary32 neighbours of every stored threshold."""
import ctypes as C

import numpy as np
import pytest

import oracle


@pytest.fixture(scope="module")
def P():
    import paper_2209_09130_amd as P
    from paper_2209_09130_amd import build as B
    import os
    if not os.path.exists(P.lib_path()):
        B.build(force=True)
    P.lib()
    return P


def lookup(spec, entries, y):
    """numpy float32 emulation of the kernel's lookup.  fmaf is emulated in float64: the product of two binary32
    numbers is exact there and the sum of it and a binary32 number rounds to binary32 once (the sum has at most
    ~80 significant bits only when the terms are far apart, where the rounding is decided by the large term;
    checked below by comparing bins against an integer-exact evaluation for sampled values)."""
    y = np.asarray(y, np.float32)
    t = (y.astype(np.float64) * np.float64(np.float32(spec.rate)) + np.float64(np.float32(spec.offset))).astype(np.float32)
    t = np.minimum(np.maximum(t, np.float32(8388608.0)), np.float32(spec.t_max))
    idx = t.view(np.uint32).astype(np.int64) - 0x4B000000
    thr = entries[idx, 0].view(np.float32)
    codes = entries[idx, 1]
    pick = np.where(y >= thr, codes >> 8, codes) & 0xFF
    return pick.astype(np.uint8).view(np.int8), idx


def oracle_codes(y, s_out):
    y = np.asarray(y, np.float32)
    return oracle.epilogue_gelu_quant(np.zeros((1, y.size), np.int32), np.zeros(y.size, np.float32), y, s_out)[0]


@pytest.mark.parametrize("s_out", [0.0247, 0.0131, 0.0052, 0.25, 1.7, 0.081])
def test_table_lookup_equals_the_definition(P, s_out):
    spec, entries = P.gelu_table_build(s_out)
    assert 2 <= spec.bins <= 2048 and entries.shape == (spec.bins, 2)
    rng = np.random.default_rng(int(s_out * 1e6))
    thr = entries[:, 0].view(np.float32)
    thr = thr[np.isfinite(thr)]
    assert thr.size >= 100                                   # a step of the code per threshold, well over a hundred of them
    near = np.concatenate([np.nextafter(thr, np.float32(-np.inf)), thr, np.nextafter(thr, np.float32(np.inf)),
                           thr - 3 * np.spacing(thr), thr + 3 * np.spacing(thr)])
    ys = np.concatenate([
        np.linspace(-12, 12, 2_000_001).astype(np.float32),
        (rng.standard_normal(1_000_000) * 0.6).astype(np.float32),
        (rng.standard_normal(200_000) * 127 * s_out).astype(np.float32),
        near.astype(np.float32),
        np.array([0.0, -0.0, 1e-30, -1e-30, 40.0, -40.0, 1e4, -1e4, 3e38, -3e38, -0.75179, -0.7517916], np.float32),
    ])
    got, idx = lookup(spec, entries, ys)
    want = oracle_codes(ys, s_out)
    bad = np.flatnonzero(got != want)
    assert bad.size == 0, (ys[bad[:5]], got[bad[:5]], want[bad[:5]], idx[bad[:5]])
    assert want.max() == 127 and (want.min() < 0 or s_out > 0.3)


def test_every_threshold_is_a_step_of_the_definition(P):
    """Each finite threshold is the first binary32 number of its bin's upper code: the number just below it has the
    bin's lower code, and the two codes differ by one step."""
    s_out = 0.0247
    spec, entries = P.gelu_table_build(s_out)
    thr = entries[:, 0].view(np.float32)
    ok = np.isfinite(thr)
    lo = (entries[ok, 1] & 0xFF).astype(np.uint8).view(np.int8).astype(int)
    hi = ((entries[ok, 1] >> 8) & 0xFF).astype(np.uint8).view(np.int8).astype(int)
    assert (np.abs(hi - lo) == 1).all()
    at = oracle_codes(thr[ok], s_out).astype(int)
    below = oracle_codes(np.nextafter(thr[ok], np.float32(-np.inf)), s_out).astype(int)
    assert np.array_equal(at, hi) and np.array_equal(below, lo)
    # bins without a threshold hold one code
    flat = entries[~ok, 1]
    assert ((flat & 0xFF) == (flat >> 8)).all()


def test_steps_too_fine_for_the_table_are_refused(P):
    with pytest.raises(P.SampError) as e:
        P.gelu_table_build(1e-5)
    assert e.value.code == -5
    with pytest.raises(P.SampError):
        P.gelu_table_build(float("nan"))
