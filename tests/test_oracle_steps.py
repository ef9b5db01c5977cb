"""Pins for the oracle's step functions (CPU only).

Each step is checked against something other than itself: numpy's own binary16
rounding, brute-force integer sums, closed forms, textbook constants, numerical
quadrature, and float64 library routines with a half-step error bound.
"""
import math
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_pairs(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            a, b = line.split()
            rows.append((float(a), float(b)))
    return rows


# ------------------------------------------------------------------ binary16
def test_half_to_float_all_bit_patterns_match_numpy():
    bits = np.arange(65536, dtype=np.uint16)
    h = bits.view(np.float16)
    got = oracle.f16_to_f32(h)
    want = h.astype(np.float32)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan].view(np.uint32), want[~nan].view(np.uint32))


def test_float_to_half_rne_matches_numpy_incl_ties_subnormals_overflow():
    rng = np.random.default_rng(0)
    # every half, every midpoint between adjacent halves, and their float neighbours
    pos = np.arange(0x7c00, dtype=np.uint16).view(np.float16).astype(np.float32)
    mids = (pos[:-1].astype(np.float64) + pos[1:].astype(np.float64)) / 2
    mids32 = mids.astype(np.float32)
    assert np.array_equal(mids32.astype(np.float64), mids)     # midpoints are exact floats
    cand = np.concatenate([pos, mids32, np.nextafter(mids32, np.float32(np.inf)),
                           np.nextafter(mids32, np.float32(-np.inf)),
                           np.array([65504, 65519.996, 65520, 65536, 1e30, np.inf, 2.0 ** -25, 2.0 ** -24 * 1.5,
                                     2.0 ** -14, 0.0], np.float32),
                           rng.standard_normal(200000).astype(np.float32) * np.float32(10),
                           (rng.standard_normal(100000) * 1e-6).astype(np.float32)])
    cand = np.concatenate([cand, -cand])
    with np.errstate(over="ignore"):
        want = cand.astype(np.float16)
    got = oracle.f32_to_f16(cand)
    assert np.array_equal(got.view(np.uint16), want.view(np.uint16))


# ------------------------------------------------------------------ quantiser
def test_quantiser_tie_table_and_clamp():
    for v, code in _read_pairs("rne_ties.txt"):
        assert oracle.quant_code(np.float32(v)) == int(code), v


def test_quantiser_invariants():
    rng = np.random.default_rng(1)
    s = np.float32(0.0371)
    x = (rng.standard_normal(50000) * 1.5).astype(np.float32)
    q = oracle.quantize_f32(x, s)
    assert q.min() >= -127 and q.max() <= 127
    assert np.array_equal(oracle.quantize_f32(-x, s), -q)                   # odd symmetry
    inside = np.abs(x) <= 127 * s
    err = np.abs(q.astype(np.float64) * float(s) - x.astype(np.float64))
    assert err[inside].max() <= float(s) / 2 * (1 + 1e-5)                   # half a step inside the range
    deq = (q.astype(np.float32) * s).astype(np.float32)
    assert np.array_equal(oracle.quantize_f32(deq, s), q)                   # idempotent
    big = np.array([1e6, -1e6], np.float32)
    assert list(oracle.quantize_f32(big, s)) == [127, -127]


def test_absmax_element_maps_to_127_and_fp16_entry_quant_is_one_multiply():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((64, 96)).astype(np.float16)
    amax = np.abs(x.astype(np.float32)).max()
    s = np.float32(amax) / np.float32(127.0)
    q = oracle.quantize_f16(x, s)
    assert np.abs(q).max() == 127
    assert abs(int(q.flat[np.argmax(np.abs(x.astype(np.float32)))])) == 127
    inv = np.float32(1.0) / s
    want = np.clip(np.rint(x.astype(np.float32) * inv), -127, 127).astype(np.int8)   # numpy rint = half to even
    assert np.array_equal(q, want)


def test_weight_quantisation_per_output_channel():
    rng = np.random.default_rng(3)
    W = (rng.standard_normal((37, 53)) * 0.02).astype(np.float16)
    W[5] = 0                      # all-zero row
    W[7] *= 30                    # a row with a much larger range must not affect the others
    Wq, s_w = oracle.quantize_weight(W)
    Wf = W.astype(np.float32)
    amax = np.abs(Wf).max(axis=1)
    assert s_w[5] == 1.0 and not Wq[5].any()
    rows = amax > 0
    assert np.array_equal(s_w[rows], (amax[rows] / np.float32(127.0)).astype(np.float32))
    assert np.array_equal(np.abs(Wq[rows]).max(axis=1), np.full(rows.sum(), 127))
    err = np.abs(Wq.astype(np.float64) * s_w[:, None].astype(np.float64) - Wf.astype(np.float64))
    assert (err <= s_w[:, None].astype(np.float64) / 2 * (1 + 1e-5)).all()
    # sign and position preserved (a transposed or mis-indexed write would break this)
    assert np.array_equal(np.sign(Wq[rows]), np.sign(np.rint(Wf[rows] / s_w[rows, None])))


# ------------------------------------------------------------------ int8 GEMM
@pytest.mark.parametrize("M,N,K", [(1, 1, 1), (3, 5, 7), (9, 4, 33), (2, 17, 129)])
def test_int8_gemm_brute_force(M, N, K):
    rng = np.random.default_rng(M * 100 + N * 10 + K)
    A = rng.integers(-127, 128, (M, K), dtype=np.int8)
    W = rng.integers(-127, 128, (N, K), dtype=np.int8)
    got = oracle.gemm_i8_i32(A, W)
    want = np.zeros((M, N), np.int64)
    for t in range(M):
        for n in range(N):
            acc = 0
            for k in range(K):
                acc += int(A[t, k]) * int(W[n, k])
            want[t, n] = acc
    assert np.array_equal(got.astype(np.int64), want)


def test_int8_gemm_extreme_values_do_not_overflow():
    K = 4096
    A = np.full((2, K), 127, np.int8)
    A[1] = -127
    W = np.full((3, K), 127, np.int8)
    W[2] = -127
    got = oracle.gemm_i8_i32(A, W)
    v = 127 * 127 * K
    assert np.array_equal(got, np.array([[v, v, -v], [-v, -v, v]], np.int32))


def test_int8_gemm_matches_int64_matmul_on_a_real_shape():
    rng = np.random.default_rng(4)
    A = rng.integers(-127, 128, (40, 768), dtype=np.int8)
    W = rng.integers(-127, 128, (96, 768), dtype=np.int8)
    assert np.array_equal(oracle.gemm_i8_i32(A, W).astype(np.int64), A.astype(np.int64) @ W.astype(np.int64).T)


# ------------------------------------------------------------------ epilogues
def test_requant_epilogue_lossless_special_case():
    # integer data, all steps 1: the INT8 GEMM + epilogue must equal the integer result clamped
    rng = np.random.default_rng(5)
    A = rng.integers(-3, 4, (6, 16), dtype=np.int8)
    W = rng.integers(-3, 4, (10, 16), dtype=np.int8)
    bias = rng.integers(-20, 21, 10).astype(np.float32)
    m, b = oracle.fold_requant(1.0, np.ones(10, np.float32), bias, 1.0)
    assert np.array_equal(m, np.ones(10, np.float32)) and np.array_equal(b, bias)
    acc = oracle.gemm_i8_i32(A, W)
    got = oracle.epilogue_requant(acc, m, b)
    want = np.clip(A.astype(np.int64) @ W.astype(np.int64).T + bias.astype(np.int64), -127, 127)
    assert np.array_equal(got.astype(np.int64), want)


def test_requant_epilogue_ties_and_per_column_tables():
    acc = np.array([[1, 3, 5, -1, -3, 255, 300]], np.int32)
    m = np.full(7, 0.5, np.float32)
    got = oracle.epilogue_requant(acc, m, np.zeros(7, np.float32))
    assert list(got[0]) == [0, 2, 2, 0, -2, 127, 127]          # .5 ties go to even, then clamp
    # distinct columns use distinct table entries
    acc = np.full((2, 4), 10, np.int32)
    got = oracle.epilogue_requant(acc, np.array([1, 2, 3, 4], np.float32), np.array([0, 1, 2, -50], np.float32))
    assert np.array_equal(got, np.array([[10, 21, 32, -10]] * 2, np.int8))


def test_fold_tables_match_exact_rational_arithmetic():
    from fractions import Fraction
    rng = np.random.default_rng(6)
    s_w = (rng.random(9) * 1e-3 + 1e-5).astype(np.float32)
    bias = rng.standard_normal(9).astype(np.float32)
    s_in, s_out = np.float32(0.0371), np.float32(0.0123)
    m, b = oracle.fold_requant(s_in, s_w, bias, s_out)
    md = oracle.fold_dequant(s_in, s_w)
    for n in range(9):
        exact_m = Fraction(float(s_in)) * Fraction(float(s_w[n])) / Fraction(float(s_out))
        exact_b = Fraction(float(bias[n])) / Fraction(float(s_out))
        exact_d = Fraction(float(s_in)) * Fraction(float(s_w[n]))
        for got, exact in ((m[n], exact_m), (b[n], exact_b), (md[n], exact_d)):
            # within one binary32 rounding (plus one binary64 rounding) of the exact value
            assert abs(Fraction(float(got)) - exact) <= abs(exact) * Fraction(1, 2 ** 23)


def _phi_quadrature(x, n=20000):
    """Phi(x) = 1/2 + integral_0^x of the normal density, composite Simpson; no erf involved."""
    t = np.linspace(0.0, x, 2 * n + 1)
    f = np.exp(-0.5 * t * t) / math.sqrt(2 * math.pi)
    h = (x - 0.0) / (2 * n)
    return 0.5 + h / 3 * (f[0] + f[-1] + 4 * f[1:-1:2].sum() + 2 * f[2:-1:2].sum())


def test_gelu_textbook_values_quadrature_and_identities():
    for x, phi in _read_pairs("normal_cdf.txt"):
        assert abs(oracle.gelu(x) - x * phi) <= 1e-9 * max(1.0, abs(x)) + 6e-8 * abs(x * phi)
    for x in np.linspace(-6, 6, 49):
        want = x * _phi_quadrature(float(x))
        assert abs(oracle.gelu(np.float32(x)) - want) <= 1e-7 + 6e-8 * abs(want)
    xs = np.random.default_rng(7).standard_normal(200).astype(np.float32) * 2
    for x in xs:                                    # x Phi(x) - (-x) Phi(-x) = x
        assert abs(oracle.gelu(x) - oracle.gelu(-x) - float(x)) <= 2e-7 * max(1.0, abs(float(x)))
    assert oracle.gelu(0.0) == 0.0
    assert oracle.gelu(30.0) == 30.0 and oracle.gelu(-30.0) == 0.0


def test_gelu_quant_epilogue_within_half_a_step_of_the_true_activation():
    rng = np.random.default_rng(8)
    acc = rng.integers(-60000, 60000, (5, 12), dtype=np.int32)
    m = (rng.random(12) * 5e-5 + 1e-5).astype(np.float32)
    bias = rng.standard_normal(12).astype(np.float32) * 0.3
    s_out = np.float32(0.0247)
    got = oracle.epilogue_gelu_quant(acc, m, bias, s_out)
    y = acc.astype(np.float64) * m.astype(np.float64) + bias.astype(np.float64)
    g = np.array([[v * _phi_quadrature(float(v)) for v in row] for row in y])
    want = np.clip(g / float(s_out), -127, 127)
    assert np.abs(got.astype(np.float64) - want).max() <= 0.5 + 1e-4
    assert (got[y < -8] == 0).all() if (y < -8).any() else True


# ------------------------------------------------------------------ LayerNorm step
def _ln64(z, g, b, eps):
    mu = z.mean(axis=1, keepdims=True)
    var = ((z - mu) ** 2).mean(axis=1, keepdims=True)
    return (z - mu) / np.sqrt(var + eps) * g + b


def test_add_ln_fp16_path_against_float64_and_torch():
    import torch
    rng = np.random.default_rng(9)
    M, H = 7, 96
    a = rng.standard_normal((M, H)).astype(np.float16)
    r = rng.standard_normal((M, H)).astype(np.float16)
    bias = rng.standard_normal(H).astype(np.float32) * 0.1
    g = (1 + 0.1 * rng.standard_normal(H)).astype(np.float32)
    be = (0.1 * rng.standard_normal(H)).astype(np.float32)
    eps = 1e-5
    got = oracle.add_ln(a, 1.0, bias, r, 1.0, g, be, eps, out_i8=False).astype(np.float64)
    z = a.astype(np.float64) + bias + r.astype(np.float64)
    want = _ln64(z, g.astype(np.float64), be.astype(np.float64), eps)
    tl = torch.nn.functional.layer_norm(torch.from_numpy(z), (H,), torch.from_numpy(g.astype(np.float64)),
                                        torch.from_numpy(be.astype(np.float64)), eps).numpy()
    assert np.abs(want - tl).max() < 1e-12
    ulp = np.maximum(np.abs(want), 2.0 ** -14) * 2.0 ** -11        # half an fp16 ulp bound
    assert (np.abs(got - want) <= ulp + 1e-6).all()


def test_add_ln_int8_paths_within_half_a_step():
    rng = np.random.default_rng(10)
    M, H = 5, 64
    a = rng.integers(-127, 128, (M, H), dtype=np.int8)
    r = rng.integers(-127, 128, (M, H), dtype=np.int8)
    s_a, s_r, s_out = np.float32(0.011), np.float32(0.037), np.float32(0.039)
    bias = rng.standard_normal(H).astype(np.float32) * 0.1
    g = (1 + 0.1 * rng.standard_normal(H)).astype(np.float32)
    be = (0.1 * rng.standard_normal(H)).astype(np.float32)
    z = a.astype(np.float64) * float(s_a) + bias + r.astype(np.float64) * float(s_r)
    want = _ln64(z, g.astype(np.float64), be.astype(np.float64), 1e-12)
    got8 = oracle.add_ln(a, s_a, bias, r, s_r, g, be, 1e-12, out_i8=True, s_out=s_out)
    assert np.abs(got8.astype(np.float64) - np.clip(want / float(s_out), -127, 127)).max() <= 0.5 + 1e-4
    got16 = oracle.add_ln(a, s_a, bias, r, s_r, g, be, 1e-12, out_i8=False).astype(np.float64)
    assert np.abs(got16 - want).max() <= 2.0 ** -9 + 1e-6          # |y| < 4 here: half ulp <= 2^-10
    # mixed operand kinds: fp16 input with int8 residual and the other way round
    a16 = (a.astype(np.float32) * s_a).astype(np.float16)
    z2 = a16.astype(np.float64) + bias + r.astype(np.float64) * float(s_r)
    want2 = _ln64(z2, g.astype(np.float64), be.astype(np.float64), 1e-12)
    got2 = oracle.add_ln(a16, 1.0, bias, r, s_r, g, be, 1e-12, out_i8=False).astype(np.float64)
    assert np.abs(got2 - want2).max() <= 2.0 ** -9 + 1e-6


def test_layernorm_invariants():
    rng = np.random.default_rng(11)
    M, H = 16, 768
    a = (rng.standard_normal((M, H)) * 3 + 1).astype(np.float16)
    zero = np.zeros((M, H), np.float16)
    one, nul = np.ones(H, np.float32), np.zeros(H, np.float32)
    y = oracle.add_ln(a, 1.0, nul, zero, 1.0, one, nul, 1e-12, out_i8=False).astype(np.float64)
    assert np.abs(y.mean(axis=1)).max() < 1e-3 and np.abs(y.var(axis=1) - 1).max() < 3e-3
    # adding a constant (through the bias) or rescaling by a power of two changes nothing
    y_shift = oracle.add_ln(a, 1.0, np.full(H, 8.0, np.float32), zero, 1.0, one, nul, 1e-12, out_i8=False)
    assert np.abs(y_shift.astype(np.float64) - y).max() <= 2.0 ** -9
    y_scale = oracle.add_ln((a.astype(np.float32) * 4).astype(np.float16), 1.0, nul, zero, 1.0, one, nul, 1e-12,
                            out_i8=False)
    assert np.array_equal(y_scale, y.astype(np.float16))
    # constant row: variance 0, eps keeps it finite, output = beta
    c = np.full((1, H), 2.5, np.float16)
    yb = oracle.add_ln(c, 1.0, nul, zero[:1], 1.0, one, np.full(H, 0.25, np.float32), 1e-5, out_i8=False)
    assert np.array_equal(yb, np.full((1, H), 0.25, np.float16))


# ------------------------------------------------------------------ fp16 GEMM
def test_fp16_gemm_against_float64_matmul():
    rng = np.random.default_rng(12)
    A = rng.standard_normal((9, 80)).astype(np.float16)
    W = (rng.standard_normal((13, 80)) * 0.05).astype(np.float16)
    bias = rng.standard_normal(13).astype(np.float32) * 0.1
    want = A.astype(np.float64) @ W.astype(np.float64).T
    got = oracle.gemm_f16(A, W, None, False).astype(np.float64)
    assert (np.abs(got - want) <= np.maximum(np.abs(want), 2.0 ** -14) * 2.0 ** -11 + 1e-7).all()
    got_b = oracle.gemm_f16(A, W, bias, False).astype(np.float64)
    wb = want + bias
    assert (np.abs(got_b - wb) <= np.maximum(np.abs(wb), 2.0 ** -14) * 2.0 ** -11 + 1e-6).all()
    got_g = oracle.gemm_f16(A, W, bias, True).astype(np.float64)
    wg = np.array([[v * _phi_quadrature(float(v)) for v in row] for row in wb])
    assert (np.abs(got_g - wg) <= np.maximum(np.abs(wg), 2.0 ** -14) * 2.0 ** -11 + 1e-6).all()


# ------------------------------------------------------------------ attention
def _softmax64(s):
    e = np.exp(s - s.max(axis=-1, keepdims=True))
    return e / e.sum(axis=-1, keepdims=True)


def test_fp16_attention_against_float64_with_several_sequences():
    rng = np.random.default_rng(13)
    heads, d = 3, 64
    H = heads * d
    cu = np.array([0, 5, 6, 23], np.int32)                 # lengths 5, 1, 17
    T = int(cu[-1])
    qkv = rng.standard_normal((T, 3 * H)).astype(np.float16)
    got = oracle.attention_f16(qkv, cu, heads).astype(np.float64)
    x = qkv.astype(np.float64)
    for b in range(3):
        sl = slice(cu[b], cu[b + 1])
        for h in range(heads):
            q = x[sl, h * d:(h + 1) * d]
            k = x[sl, H + h * d:H + (h + 1) * d]
            v = x[sl, 2 * H + h * d:2 * H + (h + 1) * d]
            P = _softmax64(q @ k.T / math.sqrt(d))
            want = P @ v
            # P is rounded to fp16 (rel 2^-11) before P.V, the result once more
            assert np.abs(got[sl, h * d:(h + 1) * d] - want).max() <= 3e-3
    # a single-key sequence attends to itself only: context = its own V exactly
    assert np.array_equal(oracle.attention_f16(qkv, cu, heads)[5], qkv[5, 2 * H:])


def test_int8_attention_softmax_codes_and_exact_integer_context():
    rng = np.random.default_rng(14)
    heads, d = 2, 64
    H = heads * d
    n = 19
    cu = np.array([0, 4, 4 + n], np.int32)
    T = int(cu[-1])
    qkv = rng.integers(-127, 128, (T, 3 * H), dtype=np.int8)
    s_q, s_k, s_v, s_p, s_ctx = map(np.float32, (0.021, 0.025, 0.02, 0.0031, 0.0067))
    ctx, Pq = oracle.attention_i8(qkv, cu, heads, s_q, s_k, s_v, s_p, s_ctx, dump_p=True)
    x = qkv[cu[1]:cu[2]].astype(np.int64)
    m_ctx = np.float32(np.float64(s_p) * np.float64(s_v) / np.float64(s_ctx))
    for h in range(heads):
        q, k, v = x[:, h * d:(h + 1) * d], x[:, H + h * d:H + (h + 1) * d], x[:, 2 * H + h * d:2 * H + (h + 1) * d]
        sc = (q @ k.T).astype(np.float64) * float(s_q) * float(s_k) / math.sqrt(d)
        P = _softmax64(sc)
        codes = Pq[h].astype(np.float64)
        assert codes.min() >= 0 and codes.max() <= 127                  # softmax codes never go negative
        assert np.abs(codes - np.clip(P / float(s_p), 0, 127)).max() <= 0.5 + 1e-3
        O = Pq[h].astype(np.int64) @ v                                     # exact integer P.V from the dumped codes
        want = np.clip(np.rint(O.astype(np.float32) * m_ctx), -127, 127).astype(np.int8)
        assert np.array_equal(ctx[cu[1]:cu[2], h * d:(h + 1) * d], want)


def test_int8_attention_closed_forms():
    heads, d = 1, 64
    H = d
    n = 8
    rng = np.random.default_rng(15)
    qkv = np.zeros((n + 1, 3 * H), np.int8)
    qkv[:, :H] = rng.integers(-50, 50, (n + 1, H))
    qkv[:n, H:2 * H] = 7                                  # identical keys: uniform probabilities 1/n
    qkv[:, 2 * H:] = rng.integers(-127, 128, (n + 1, H))
    cu = np.array([0, n, n + 1], np.int32)
    s_p, s_v, s_ctx = np.float32(1 / 127 / 4), np.float32(0.02), np.float32(0.004)
    ctx, Pq = oracle.attention_i8(qkv, cu, heads, 0.02, 0.02, s_v, s_p, s_ctx, dump_p=True)
    code = int(np.rint(np.float32(1.0 / n) * (np.float32(1.0) / s_p)))
    m_ctx = np.float32(np.float64(s_p) * np.float64(s_v) / np.float64(s_ctx))
    vsum = qkv[:n, 2 * H:].astype(np.int64).sum(axis=0)
    want = np.clip(np.rint((code * vsum).astype(np.float32) * m_ctx), -127, 127).astype(np.int8)
    for i in range(n):
        assert np.array_equal(ctx[i], want)
    # the last sequence has a single key: probability 1, code rne(1/s_p) clamped to 127
    assert Pq.shape == (1, 1, 1) and Pq[0, 0, 0] == 127
    want1 = np.clip(np.rint((127 * qkv[n, 2 * H:].astype(np.int64)).astype(np.float32) * m_ctx), -127, 127)
    assert np.array_equal(ctx[n].astype(np.int64), want1.astype(np.int64))


def test_int8_attention_unsigned_softmax_codes():
    """Variant that spends all 256 codes on [0, 1] (Section 4.2 / Appendix B name the idle negative half of the
    symmetric code as the main accuracy loss): codes are rne(P / s) clamped to [0, 255]; everything else is unchanged."""
    rng = np.random.default_rng(17)
    heads, d = 2, 64
    H = heads * d
    n = 23
    cu = np.array([0, 3, 3 + n], np.int32)
    qkv = rng.integers(-127, 128, (int(cu[-1]), 3 * H), dtype=np.int8)
    s_q, s_k, s_v, s_ctx = map(np.float32, (0.021, 0.025, 0.02, 0.0067))
    x = qkv[cu[1]:cu[2]].astype(np.int64)
    P64 = [_softmax64((x[:, h * d:(h + 1) * d] @ x[:, H + h * d:H + (h + 1) * d].T).astype(np.float64)
                      * float(s_q) * float(s_k) / math.sqrt(d)) for h in range(heads)]
    absmax = max(p.max() for p in P64) * 0.8                       # some probabilities clamp
    s_signed, s_unsigned = np.float32(absmax / 127), np.float32(absmax / 255)
    ctx, Pu = oracle.attention_i8(qkv, cu, heads, s_q, s_k, s_v, s_unsigned, s_ctx, dump_p=True, p_unsigned=True)
    _, Ps = oracle.attention_i8(qkv, cu, heads, s_q, s_k, s_v, s_signed, s_ctx, dump_p=True)
    assert Pu.dtype == np.uint8 and Pu.max() == 255 and Ps.max() == 127
    m_ctx = np.float32(np.float64(s_unsigned) * np.float64(s_v) / np.float64(s_ctx))
    err_u, err_s = [], []
    for h in range(heads):
        codes = Pu[h].astype(np.float64)
        assert np.abs(codes - np.clip(P64[h] / float(s_unsigned), 0, 255)).max() <= 0.5 + 1e-3
        v = x[:, 2 * H + h * d:2 * H + (h + 1) * d]
        O = Pu[h].astype(np.int64) @ v                                   # exact integer P.V from the dumped codes
        want = np.clip(np.rint(O.astype(np.float32) * m_ctx), -127, 127).astype(np.int8)
        assert np.array_equal(ctx[cu[1]:cu[2], h * d:(h + 1) * d], want)
        inside = P64[h] < absmax * 0.99
        err_u.append(np.abs(codes * float(s_unsigned) - P64[h])[inside])
        err_s.append(np.abs(Ps[h].astype(np.float64) * float(s_signed) - P64[h])[inside])
    # twice as many levels over the same range: half the rounding error
    ratio = np.concatenate(err_u).mean() / np.concatenate(err_s).mean()
    assert 0.4 <= ratio <= 0.6
    # a single-key sequence has probability 1: the top code
    one = rng.integers(-127, 128, (1, 3 * H), dtype=np.int8)
    _, P1 = oracle.attention_i8(one, np.array([0, 1], np.int32), heads, s_q, s_k, s_v, np.float32(1 / 255), s_ctx,
                                dump_p=True, p_unsigned=True)
    assert P1.shape == (heads, 1, 1) and (P1 == 255).all()


def test_int8_attention_with_binary16_softmax_output():
    """The variant that keeps the softmax output out of the 8-bit grid (Section 4.2 / Appendix B name its quantisation
    as the accuracy problem of a fully quantised attention block): P is rounded to binary16, V stays integer codes.
    Pins: brute force through float64 probabilities rounded by numpy to float16 and summed in exact integer arithmetic;
    closed forms (one key; identical keys with a power-of-two and a non-power-of-two count); the error against the
    unrounded context must be that of the final rounding alone, and below the 8-bit softmax variant's."""
    from fractions import Fraction
    rng = np.random.default_rng(19)
    heads, d = 2, 64
    H = heads * d
    n = 37
    cu = np.array([0, 2, 2 + n], np.int32)
    qkv = rng.integers(-127, 128, (int(cu[-1]), 3 * H), dtype=np.int8)
    s_q, s_k, s_v, s_ctx = map(np.float32, (0.021, 0.025, 0.02, 0.0067))
    m = np.float32(np.float64(s_v) / np.float64(s_ctx))
    ctx = oracle.attention_i8_p16(qkv, cu, heads, s_q, s_k, s_v, s_ctx)
    x = qkv[cu[1]:cu[2]].astype(np.int64)
    differ, ideal_err, int8_err = 0, [], []
    P_all = []
    for h in range(heads):
        q, k, v = x[:, h * d:(h + 1) * d], x[:, H + h * d:H + (h + 1) * d], x[:, 2 * H + h * d:2 * H + (h + 1) * d]
        P = _softmax64((q @ k.T).astype(np.float64) * float(s_q) * float(s_k) / math.sqrt(d))
        P_all.append(P)
        # float16 values are multiples of 2^-24: the sum over keys as an exact integer, rounded once to float32
        P24 = np.rint(P.astype(np.float16).astype(np.float64) * 2.0 ** 24).astype(np.int64)
        O = (P24 @ v).astype(np.float64) * 2.0 ** -24                      # |sum| < 2^31: exact in float64
        want = np.clip(np.rint(O.astype(np.float32) * m), -127, 127).astype(np.int64)
        got = ctx[cu[1]:cu[2], h * d:(h + 1) * d].astype(np.int64)
        # the oracle reaches P through binary32 (e * rS) before binary16: a few P differ by one float16 ulp
        assert np.abs(got - want).max() <= 1
        differ += int((got != want).sum())
        ideal = (P @ v) * float(m)
        ideal_err.append(np.abs(got - np.clip(ideal, -127, 127)))
    assert differ <= 0.01 * n * H
    # each P16 is within 2^-12 relative of P and the P of a row sum to 1: the unrounded context moves by at most
    # 127 * m * 2^-12 steps (twice that allowed for the binary32 detour), then comes the one final rounding
    assert np.concatenate(ideal_err).max() <= 0.5 + 127 * float(m) * 2.0 ** -11
    # the 8-bit softmax code with the best static step is much further from the ideal context
    s_p = np.float32(max(p.max() for p in P_all) / 127)
    ctx8 = oracle.attention_i8(qkv, cu, heads, s_q, s_k, s_v, s_p, s_ctx)
    for h in range(heads):
        v = x[:, 2 * H + h * d:2 * H + (h + 1) * d]
        ideal = np.clip((P_all[h] @ v) * float(m), -127, 127)
        int8_err.append(np.abs(ctx8[cu[1]:cu[2], h * d:(h + 1) * d].astype(np.float64) - ideal))
    assert np.concatenate(ideal_err).mean() < 0.8 * np.concatenate(int8_err).mean()

    # one key: P = 1, context = rne(v * m)
    first = qkv[:2].copy()
    one = oracle.attention_i8_p16(first[:1], np.array([0, 1], np.int32), heads, s_q, s_k, s_v, s_ctx)
    assert np.array_equal(one[0], np.clip(np.rint(first[0, 2 * H:].astype(np.float32) * m), -127, 127).astype(np.int8))
    # identical keys: P = 1/n for every key; n = 64 is exact in binary16, n = 3 and 48 round twice (binary32, binary16;
    # leaving out the binary16 rounding changes some of these contexts)
    for cnt in (64, 3, 48):
        z = np.zeros((cnt, 3 * H), np.int8)
        z[:, :H] = rng.integers(-50, 50, (cnt, H))
        z[:, H:2 * H] = 5
        z[:, 2 * H:] = rng.integers(-127, 128, (cnt, H))
        got = oracle.attention_i8_p16(z, np.array([0, cnt], np.int32), heads, s_q, s_k, s_v, s_ctx)
        p16 = Fraction(float(np.float16(np.float32(1.0) / np.float32(cnt))))
        vsum = z[:, 2 * H:].astype(np.int64).sum(axis=0)
        want = [int(np.clip(np.rint(np.float32(float(p16 * int(t))) * m), -127, 127)) for t in vsum]
        for i in range(cnt):
            assert got[i].astype(np.int64).tolist() == want


def test_attention_sequences_are_independent():
    rng = np.random.default_rng(16)
    heads, d = 2, 64
    H = heads * d
    qkv = rng.integers(-127, 128, (30, 3 * H), dtype=np.int8)
    sc = (0.021, 0.025, 0.02, 0.0031, 0.0067)
    both = oracle.attention_i8(qkv, np.array([0, 11, 30], np.int32), heads, *sc)
    first = oracle.attention_i8(qkv[:11], np.array([0, 11], np.int32), heads, *sc)
    second = oracle.attention_i8(qkv[11:], np.array([0, 19], np.int32), heads, *sc)
    assert np.array_equal(both, np.concatenate([first, second]))
    qf = rng.standard_normal((30, 3 * H)).astype(np.float16)
    bothf = oracle.attention_f16(qf, np.array([0, 11, 30], np.int32), heads)
    assert np.array_equal(bothf[:11], oracle.attention_f16(qf[:11], np.array([0, 11], np.int32), heads))


# ------------------------------------------------------------------ embedding kernel
def _emb(rng, V=50, G=2, Pn=16, H=128):
    return {"tok": (rng.standard_normal((V, H)) * 0.5).astype(np.float16), "seg": (rng.standard_normal((G, H)) * 0.5).astype(np.float16),
            "pos": (rng.standard_normal((Pn, H)) * 0.5).astype(np.float16),
            "gamma": (1 + 0.2 * rng.standard_normal(H)).astype(np.float32), "beta": (0.3 * rng.standard_normal(H)).astype(np.float32),
            "eps": 1e-12}


def test_embedding_kernel_against_torch_embedding_and_layer_norm():
    """Section 3.1: token + segment + position embeddings, then BERT's LayerNorm; checked against the library
    routines in float64 (fp16 output: half an ulp; int8 output: half a step)."""
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(41)
    emb = _emb(rng)
    n = 13
    ids = rng.integers(0, 50, n).astype(np.int32)
    seg = rng.integers(0, 2, n).astype(np.int32)
    t64 = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    z = (torch.nn.functional.embedding(torch.from_numpy(ids.astype(np.int64)), t64(emb["tok"]))
         + torch.nn.functional.embedding(torch.from_numpy(seg.astype(np.int64)), t64(emb["seg"])) + t64(emb["pos"])[:n])
    want = torch.nn.functional.layer_norm(z, (128,), t64(emb["gamma"]), t64(emb["beta"]), 1e-12).numpy()
    got = oracle.embed_ln(emb, ids, seg, out_i8=False).astype(np.float64)
    assert np.abs(got - want).max() <= np.abs(want).max() * 2.0 ** -11 + 1e-6
    s_out = np.float32(np.abs(want).max() / 127)
    codes = oracle.embed_ln(emb, ids, seg, out_i8=True, s_out=s_out).astype(np.float64)
    assert np.abs(codes - want / float(s_out)).max() <= 0.5 + 1e-3 and np.abs(codes).max() == 127
    # no segment ids = segment 0
    assert np.array_equal(oracle.embed_ln(emb, ids, None, False), oracle.embed_ln(emb, ids, np.zeros(n, np.int32), False))


def test_embedding_kernel_closed_forms_and_id_clamping():
    rng = np.random.default_rng(42)
    emb = _emb(rng)
    # a constant row has zero variance: with eps > 0 the output is beta exactly
    flat = dict(emb, tok=np.full((50, 128), 0.25, np.float16), seg=np.full((2, 128), -0.5, np.float16),
                pos=np.full((16, 128), 1.0, np.float16), eps=1e-5)
    got = oracle.embed_ln(flat, np.array([3, 4], np.int32), None, False)
    assert np.array_equal(got, np.tile(emb["beta"].astype(np.float16), (2, 1)))
    # the position is the index inside the sequence: the same token at two positions differs by the position rows
    same = oracle.embed_ln(dict(emb, gamma=np.ones(128, np.float32), beta=np.zeros(128, np.float32)),
                           np.array([7, 7], np.int32), None, False)
    assert not np.array_equal(same[0], same[1])
    # ids outside the tables are clamped into them
    a = oracle.embed_ln(emb, np.array([-5, 999], np.int32), np.array([9, -1], np.int32), False)
    b = oracle.embed_ln(emb, np.array([0, 49], np.int32), np.array([1, 0], np.int32), False)
    assert np.array_equal(a, b)


def test_encoder_with_embedding_entry_equals_embedding_then_encoder_for_fp16_entry():
    """With an FP16 first block the Embedding kernel's fp16 output IS the encoder input; with an INT8 first block the
    kernel quantises its binary32 LayerNorm value directly (Section 3.2: INT8 between Embedding and Encoder)."""
    import samp_workloads as W
    w = W.Workload("emb", 2, 128, 2, 256, 3, 12, (W.FFN_INT8, W.FULL_INT8), varlen=True, min_len=1, plain_params=False,
                   calib_batch=2, calib_seq=12)
    wts = W.make_weights(w)
    _, lens, _ = W.make_hidden(w)
    emb = W.make_embedding(w, vocab=64)
    ids, seg = W.make_ids(w, vocab=64)
    hid = np.zeros((w.batch, w.seq, w.hidden), np.float16)
    for b in range(w.batch):
        hid[b, :lens[b]] = oracle.embed_ln(emb, ids[b, :lens[b]], seg[b, :lens[b]], False)
    cfg = (w.layers, w.hidden, w.heads, w.ffn, w.ln_eps)
    sc = oracle.calibrate(*cfg, wts, hid[:2])
    enc = oracle.Encoder(*cfg, w.modes, wts, sc)
    assert np.array_equal(enc.forward_ids(emb, ids, seg, lens), enc.forward(hid, lens))
    enc.close()
    enc8 = oracle.Encoder(*cfg, (W.FULL_INT8, W.FULL_INT8), wts, sc)
    out_ids = enc8.forward_ids(emb, ids, seg, lens)
    x0 = oracle.embed_ln(emb, ids[0, :lens[0]], seg[0, :lens[0]], True, sc[0, 0])
    _, taps = enc8.forward(hid[:1], lens[:1], tap_layer=0)
    # same codes except where the fp16 rounding of the hand-over moved a value across a rounding boundary
    assert (x0 != taps["x"]).mean() < 0.02 and np.abs(x0.astype(int) - taps["x"].astype(int)).max() <= 1
    assert not out_ids[0, lens[0]:].any()
    enc8.close()


# ------------------------------------------------------------------ classification target
def test_classification_target_against_torch_linear_layers_and_closed_forms():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(51)
    B, S, H, Cn = 4, 6, 128, 5
    hid = rng.standard_normal((B, S, H)).astype(np.float16)
    wp = (rng.standard_normal((H, H)) * 0.1).astype(np.float16)
    bp = (rng.standard_normal(H) * 0.1).astype(np.float32)
    wc = (rng.standard_normal((Cn, H)) * 0.1).astype(np.float16)
    bc = (rng.standard_normal(Cn) * 0.1).astype(np.float32)
    got = oracle.classify(hid, wp, bp, wc, bc)
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    pooled = torch.tanh(torch.nn.functional.linear(t(hid[:, 0]), t(wp), t(bp)))
    want = torch.nn.functional.linear(pooled, t(wc), t(bc)).numpy()
    assert np.abs(got - want).max() < 1e-12
    # only the first token matters
    other = hid.copy(); other[:, 1:] = 0
    assert np.array_equal(oracle.classify(other, wp, bp, wc, bc), got)
    # zero pooler weights: pooled = tanh(b_p), logits = W_c tanh(b_p) + b_c for every sequence
    z = oracle.classify(hid, np.zeros_like(wp), bp, wc, bc)
    assert np.allclose(z, np.tanh(bp.astype(np.float64)) @ wc.astype(np.float64).T + bc, atol=1e-14)
    # a large pre-activation saturates tanh: identity-like pooler with a big bias gives logits = sum of W_c rows + b_c
    sat = oracle.classify(hid, np.zeros_like(wp), np.full(H, 50.0, np.float32), wc, bc)
    assert np.allclose(sat, wc.astype(np.float64).sum(axis=1) + bc, atol=1e-12)
