"""Pins for the oracle's encoder: unquantised reference against PyTorch's own
TransformerEncoderLayer, calibration against an independent float64 numpy
forward, the wiring of every precision mode re-derived from the step functions,
sequence independence, padding, and closeness of the quantised modes to the
unquantised model.  CPU only.
"""
import math
from dataclasses import replace

import numpy as np
import pytest

import oracle
import samp_workloads as W
from samp_workloads import FP16, MHA_INT8, FFN_INT8, FULL_INT8, P_UNSIGNED, P_FP16


def small(layers=2, modes=FULL_INT8, batch=3, seq=24, varlen=True, **kw):
    if isinstance(modes, int):
        modes = (modes,) * layers
    return W.Workload("small", layers, 128, 2, 256, batch, seq, tuple(modes), varlen=varlen, min_len=3,
                      plain_params=False, calib_batch=4, calib_seq=24, **kw)


def args(w):
    return (w.layers, w.hidden, w.heads, w.ffn, w.ln_eps)


def make(w):
    wts = W.make_weights(w)
    hid, lens, mask = W.make_hidden(w)
    sc = oracle.calibrate(*args(w), wts, W.make_calibration_batch(w))
    return wts, hid, lens, sc


# ------------------------------------------------------------------ reference vs PyTorch
def test_reference_forward_matches_torch_transformer_encoder_layer():
    import torch
    w = small(layers=2, ln_eps=1e-5)
    wts = W.make_weights(w)
    hid, lens, _ = W.make_hidden(w)
    got, _ = oracle.reference_forward(*args(w), wts, hid, lens)
    x = torch.from_numpy(hid.astype(np.float64))
    pad = torch.from_numpy(np.arange(w.seq)[None, :] >= lens[:, None])
    for lw in wts:
        layer = torch.nn.TransformerEncoderLayer(w.hidden, w.heads, w.ffn, dropout=0.0, activation="gelu",
                                                 layer_norm_eps=w.ln_eps, batch_first=True, norm_first=False,
                                                 dtype=torch.float64)
        layer.eval()
        t = lambda k: torch.from_numpy(lw[k].astype(np.float64))
        with torch.no_grad():
            layer.self_attn.in_proj_weight.copy_(t("w_qkv")); layer.self_attn.in_proj_bias.copy_(t("b_qkv"))
            layer.self_attn.out_proj.weight.copy_(t("w_o")); layer.self_attn.out_proj.bias.copy_(t("b_o"))
            layer.linear1.weight.copy_(t("w_ffn1")); layer.linear1.bias.copy_(t("b_ffn1"))
            layer.linear2.weight.copy_(t("w_ffn2")); layer.linear2.bias.copy_(t("b_ffn2"))
            layer.norm1.weight.copy_(t("ln1_g")); layer.norm1.bias.copy_(t("ln1_b"))
            layer.norm2.weight.copy_(t("ln2_g")); layer.norm2.bias.copy_(t("ln2_b"))
            # plain (unfused) path so that padded keys are masked, padded rows computed but ignored
            q = x
            a = layer.self_attn(q, q, q, key_padding_mask=pad, need_weights=False)[0]
            h1 = layer.norm1(q + a)
            x = layer.norm2(h1 + layer.linear2(torch.nn.functional.gelu(layer.linear1(h1))))
    want = x.numpy()
    for b in range(w.batch):
        n = lens[b]
        assert np.abs(got[b, :n] - want[b, :n]).max() < 1e-9
        assert not got[b, n:].any()


# ------------------------------------------------------------------ calibration
def _np_layer(x, lw, heads, eps):
    """Independent float64 layer (vectorised numpy); returns output and the ten calibrated tensors."""
    H = x.shape[1]
    d = H // heads
    f = lambda k: lw[k].astype(np.float64)
    qkv = x @ f("w_qkv").T + f("b_qkv")
    q, k, v = qkv[:, :H], qkv[:, H:2 * H], qkv[:, 2 * H:]
    ctx = np.zeros_like(x)
    pmax = 0.0
    for h in range(heads):
        s = q[:, h * d:(h + 1) * d] @ k[:, h * d:(h + 1) * d].T / math.sqrt(d)
        e = np.exp(s - s.max(axis=1, keepdims=True))
        P = e / e.sum(axis=1, keepdims=True)
        pmax = max(pmax, P.max())
        ctx[:, h * d:(h + 1) * d] = P @ v[:, h * d:(h + 1) * d]
    ao = ctx @ f("w_o").T

    def ln(z, g, b):
        mu = z.mean(axis=1, keepdims=True)
        var = ((z - mu) ** 2).mean(axis=1, keepdims=True)
        return (z - mu) / np.sqrt(var + eps) * f(g) + f(b)
    h1 = ln(ao + f("b_o") + x, "ln1_g", "ln1_b")
    pre = h1 @ f("w_ffn1").T + f("b_ffn1")
    g = 0.5 * pre * (1 + np.vectorize(math.erf)(pre / math.sqrt(2)))
    f2 = g @ f("w_ffn2").T
    y = ln(f2 + f("b_ffn2") + h1, "ln2_g", "ln2_b")
    am = [np.abs(t).max() for t in (x, q, k, v)] + [pmax] + [np.abs(t).max() for t in (ctx, ao, h1, g, f2)]
    return y, np.array(am)


def test_calibration_is_absmax_over_127_of_the_unquantised_tensors():
    w = small(layers=2)
    wts = W.make_weights(w)
    cal = W.make_calibration_batch(w)
    sc = oracle.calibrate(*args(w), wts, cal)
    assert sc.shape == (2, 10) and sc.dtype == np.float32
    want = np.zeros((2, 10))
    for b in range(cal.shape[0]):
        x = cal[b].astype(np.float64)
        for l in range(2):
            x, am = _np_layer(x, wts[l], w.heads, w.ln_eps)
            want[l] = np.maximum(want[l], am)
    assert np.abs(sc.astype(np.float64) * 127 / want - 1).max() < 1e-6
    # layer-0 input step is exactly the batch's absmax / 127 in binary32; softmax step is at most 1/127
    assert sc[0, 0] == np.float32(np.abs(cal.astype(np.float32)).max()) / np.float32(127)
    assert (sc[:, 4] <= np.float32(1) / np.float32(127)).all() and (sc > 0).all()


# ------------------------------------------------------------------ wiring of every mode from the step functions
def _replay_layer(t, lw, s, mode, heads, eps, next_sx):
    """Recompute one layer from its tapped input with the step functions, following Section 3.2:
    which tensors are int8, where the biases enter, which tensor is the residual, which step quantises."""
    sx, sq, sk, sv, sp, sctx, sao, sh1, sf1, sf2 = [np.float32(v) for v in s]
    H = lw["w_o"].shape[0]
    n = t["x"].shape[0]
    cu = np.array([0, n], np.int32)
    out = {}
    x = t["x"]
    if mode & 1:
        assert x.dtype == np.int8
        Wq, sw = oracle.quantize_weight(lw["w_qkv"])
        m = np.empty(3 * H, np.float32); b = np.empty(3 * H, np.float32)
        for part, so in enumerate((sq, sk, sv)):
            sl = slice(part * H, (part + 1) * H)
            m[sl], b[sl] = oracle.fold_requant(sx, sw[sl], lw["b_qkv"][sl], so)
        out["qkv"] = oracle.epilogue_requant(oracle.gemm_i8_i32(x, Wq), m, b)
        if mode & P_FP16:
            out["ctx"] = oracle.attention_i8_p16(out["qkv"], cu, heads, sq, sk, sv, sctx)
        else:
            out["ctx"] = oracle.attention_i8(out["qkv"], cu, heads, sq, sk, sv, sp, sctx, p_unsigned=bool(mode & 4))
        Wq, sw = oracle.quantize_weight(lw["w_o"])
        m, b = oracle.fold_requant(sctx, sw, None, sao)
        out["attn_out"] = oracle.epilogue_requant(oracle.gemm_i8_i32(out["ctx"], Wq), m, b)
    else:
        assert x.dtype == np.float16
        out["qkv"] = oracle.gemm_f16(x, lw["w_qkv"], lw["b_qkv"], False)
        out["ctx"] = oracle.attention_f16(out["qkv"], cu, heads)
        out["attn_out"] = oracle.gemm_f16(out["ctx"], lw["w_o"], None, False)
    out["h1"] = oracle.add_ln(out["attn_out"], sao, lw["b_o"], x, sx, lw["ln1_g"], lw["ln1_b"], eps,
                              out_i8=bool(mode & 2), s_out=sh1)
    if mode & 2:
        Wq, sw = oracle.quantize_weight(lw["w_ffn1"])
        out["ffn_mid"] = oracle.epilogue_gelu_quant(oracle.gemm_i8_i32(out["h1"], Wq), oracle.fold_dequant(sh1, sw),
                                                    lw["b_ffn1"], sf1)
        Wq, sw = oracle.quantize_weight(lw["w_ffn2"])
        m, b = oracle.fold_requant(sf1, sw, None, sf2)
        out["ffn_out"] = oracle.epilogue_requant(oracle.gemm_i8_i32(out["ffn_mid"], Wq), m, b)
    else:
        out["ffn_mid"] = oracle.gemm_f16(out["h1"], lw["w_ffn1"], lw["b_ffn1"], True)
        out["ffn_out"] = oracle.gemm_f16(out["ffn_mid"], lw["w_ffn2"], None, False)
    out["y"] = oracle.add_ln(out["ffn_out"], sf2, lw["b_ffn2"], out["h1"], sh1, lw["ln2_g"], lw["ln2_b"], eps,
                             out_i8=next_sx is not None, s_out=next_sx if next_sx is not None else 1.0)
    return out


@pytest.mark.parametrize("modes", [(FULL_INT8, FULL_INT8), (FFN_INT8, FFN_INT8), (MHA_INT8, MHA_INT8),
                                   (FP16, FP16), (FP16, FULL_INT8), (FULL_INT8, FP16), (FFN_INT8, MHA_INT8),
                                   (MHA_INT8, FFN_INT8), (FULL_INT8 | P_UNSIGNED, MHA_INT8 | P_UNSIGNED),
                                   (FULL_INT8, FULL_INT8 | P_UNSIGNED), (FULL_INT8 | P_FP16, MHA_INT8 | P_FP16),
                                   (FP16, FULL_INT8 | P_FP16)])
def test_every_mode_is_wired_as_section_3_2_says(modes):
    w = small(layers=2, modes=modes, batch=1)
    wts, hid, lens, sc = make(w)
    enc = oracle.Encoder(*args(w), w.modes, wts, sc)
    n = int(lens[0])
    for layer in range(2):
        out, t = enc.forward(hid, lens, tap_layer=layer)
        mode = modes[layer]
        kinds = {"x": mode & 1, "qkv": mode & 1, "ctx": mode & 1, "attn_out": mode & 1,
                 "h1": mode & 2, "ffn_mid": mode & 2, "ffn_out": mode & 2}
        for k, q in kinds.items():                         # int8 between kernels exactly inside quantised blocks
            assert t[k].dtype == (np.int8 if q else np.float16), k
        next_sx = sc[1, 0] if (layer == 0 and modes[1] & 1) else None
        rep = _replay_layer(t, wts[layer], sc[layer], mode, w.heads, w.ln_eps, next_sx)
        for k, v in rep.items():
            assert np.array_equal(v, t[k]), (modes, layer, k)
        if layer == 0:
            # entry: layer 0's input is the hidden state itself, quantised only if its MHA is INT8
            want_x = oracle.quantize_f16(hid[0, :n], sc[0, 0]) if mode & 1 else hid[0, :n]
            assert np.array_equal(t["x"], want_x)
        else:
            assert t["y"].dtype == np.float16                     # the last step never quantises
            assert np.array_equal(t["y"], out[0, :n])
    enc.close()


def test_quantised_ffn_block_is_identical_in_fully_quant_and_ffn_only_modes():
    # same int8 FFN input => same FFN codes, whatever the attention block's precision was
    w = small(layers=1, modes=FULL_INT8, batch=1)
    wts, hid, lens, sc = make(w)
    full = oracle.Encoder(*args(w), (FULL_INT8,), wts, sc)
    _, t = full.forward(hid, lens, tap_layer=0)
    rep = _replay_layer({"x": hid[0, :lens[0]]}, wts[0], sc[0], FFN_INT8, w.heads, w.ln_eps, None)
    # feed the Fully-Quant layer's h1 codes through the FFN-only layer's FFN steps
    Wq, sw = oracle.quantize_weight(wts[0]["w_ffn1"])
    mid = oracle.epilogue_gelu_quant(oracle.gemm_i8_i32(t["h1"], Wq), oracle.fold_dequant(sc[0, 7], sw),
                                     wts[0]["b_ffn1"], sc[0, 8])
    assert np.array_equal(mid, t["ffn_mid"])
    assert rep["ffn_mid"].dtype == np.int8 and rep["y"].dtype == np.float16
    full.close()


# ------------------------------------------------------------------ independence, padding, chaining
@pytest.mark.parametrize("mode", [FP16, MHA_INT8, FFN_INT8, FULL_INT8])
def test_sequences_are_independent_and_padding_is_inert(mode):
    w = small(layers=2, modes=mode, batch=4)
    wts, hid, lens, sc = make(w)
    enc = oracle.Encoder(*args(w), w.modes, wts, sc)
    out = enc.forward(hid, lens)
    for b in range(w.batch):
        n = int(lens[b])
        assert not out[b, n:].any()                                # padded rows come back as zeros
        alone = enc.forward(hid[b:b + 1, :n].copy(), np.array([n], np.int32))
        assert np.array_equal(alone[0], out[b, :n])                # alone, unpadded: bit identical
    hid2 = hid.copy()
    for b in range(w.batch):
        hid2[b, lens[b]:] = 77.0                                   # different garbage in the padding
    assert np.array_equal(enc.forward(hid2, lens), out)
    assert np.array_equal(enc.forward(hid, lens, nthreads=1), out)  # thread count does not matter
    enc.close()


def test_bad_lengths_are_rejected():
    w = small(layers=1, modes=FP16, batch=2)
    wts, hid, lens, sc = make(w)
    enc = oracle.Encoder(*args(w), w.modes, wts, sc)
    with pytest.raises(ValueError):
        enc.forward(hid, np.array([0, 5], np.int32))
    with pytest.raises(ValueError):
        enc.forward(hid, np.array([5, w.seq + 1], np.int32))
    enc.close()


def test_two_layers_equal_two_single_layer_runs_when_the_hand_over_is_fp16():
    w = small(layers=2, modes=(FFN_INT8, FFN_INT8), batch=2)
    wts, hid, lens, sc = make(w)
    both = oracle.Encoder(*args(w), w.modes, wts, sc)
    one = oracle.Encoder(1, w.hidden, w.heads, w.ffn, w.ln_eps, (FFN_INT8,), wts[:1], sc[:1])
    two = oracle.Encoder(1, w.hidden, w.heads, w.ffn, w.ln_eps, (FFN_INT8,), wts[1:], sc[1:])
    assert np.array_equal(two.forward(one.forward(hid, lens), lens), both.forward(hid, lens))
    for e in (both, one, two):
        e.close()


# ------------------------------------------------------------------ closeness to the unquantised model
def test_fp16_mode_tracks_the_unquantised_reference():
    w = small(layers=2, modes=FP16)
    wts, hid, lens, sc = make(w)
    enc = oracle.Encoder(*args(w), w.modes, wts, None)            # no scales needed without INT8 blocks
    out = enc.forward(hid, lens).astype(np.float64)
    ref, _ = oracle.reference_forward(*args(w), wts, hid, lens)
    assert np.abs(out - ref).max() < 1e-2 and np.abs(out - ref).mean() < 1e-3
    enc.close()


@pytest.mark.parametrize("mode,cos_min", [(FFN_INT8, 0.995), (MHA_INT8, 0.995), (FULL_INT8, 0.99)])
def test_quantised_modes_stay_close_to_the_unquantised_reference(mode, cos_min):
    # sanity bound only: post-training quantisation error depends on the data (Section 4.2)
    w = W.bert_base("one", 1, 2, 48, mode, plain_params=False, calib_batch=4, calib_seq=48)
    wts, hid, lens, sc = make(w)
    enc = oracle.Encoder(*args(w), w.modes, wts, sc)
    out = enc.forward(hid, lens).astype(np.float64).ravel()
    ref = oracle.reference_forward(*args(w), wts, hid, lens)[0].ravel()
    cos = out @ ref / np.linalg.norm(out) / np.linalg.norm(ref)
    assert cos > cos_min
    assert np.abs(out - ref).mean() < 0.05
    enc.close()
