"""ctypes front end of the CPU oracle (oracle/samp_oracle.c).

TEST INFRASTRUCTURE ONLY: tests/, __graft_entry__.smoke() and the cpu_baseline
leg of bench.py may import this package; the product package never does.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from typing import Dict, List, Optional, Sequence

import numpy as np

_DIR = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_DIR, "samp_oracle.c")
_LIB = os.path.join(_DIR, "liboracle.so")

SCALE_FIELDS = ("x", "q", "k", "v", "p", "ctx", "attn_out", "ffn_in", "ffn_mid", "ffn_out")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc.  -ffp-contract=off: no silent fused multiply-adds."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O3", "-march=x86-64-v3", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-fvisibility=hidden", "-shared", "-fPIC", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Config(C.Structure):
    _fields_ = [("layers", C.c_int32), ("hidden", C.c_int32), ("heads", C.c_int32), ("ffn", C.c_int32),
                ("ln_eps", C.c_float)]


_WFIELDS = ("w_qkv", "w_o", "w_ffn1", "w_ffn2", "b_qkv", "b_o", "b_ffn1", "b_ffn2",
            "ln1_g", "ln1_b", "ln2_g", "ln2_b")


class _LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WFIELDS]


class _LayerScales(C.Structure):
    _fields_ = [(n, C.c_float) for n in SCALE_FIELDS]


class _Taps(C.Structure):
    _fields_ = [("layer", C.c_int32)] + [(n, C.c_void_p) for n in
                                         ("x", "qkv", "ctx", "attn_out", "h1", "ffn_mid", "ffn_out", "y")]


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.orc_gelu.restype = C.c_float
        _lib.orc_gelu.argtypes = [C.c_float]
        _lib.orc_quant_code.restype = C.c_int
        _lib.orc_quant_code.argtypes = [C.c_float]
        _lib.orc_encoder_create.restype = C.c_void_p
        _lib.orc_max_threads.restype = C.c_int
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def _f16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16, a.dtype
    return a


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def max_threads() -> int:
    return int(lib().orc_max_threads())


# ---------------------------------------------------------------- step functions
def f16_to_f32(x: np.ndarray) -> np.ndarray:
    x = _f16(x)
    out = np.empty(x.shape, np.float32)
    lib().orc_f16_to_f32(_p(x), _p(out), C.c_size_t(x.size))
    return out


def f32_to_f16(x: np.ndarray) -> np.ndarray:
    x = _f32(x)
    out = np.empty(x.shape, np.float16)
    lib().orc_f32_to_f16(_p(x), _p(out), C.c_size_t(x.size))
    return out


def quant_code(v: float) -> int:
    return int(lib().orc_quant_code(C.c_float(v)))


def gelu(y: float) -> float:
    return float(lib().orc_gelu(C.c_float(y)))


def quantize_f16(x: np.ndarray, s: float) -> np.ndarray:
    x = _f16(x)
    out = np.empty(x.shape, np.int8)
    lib().orc_quantize_f16(_p(x), C.c_size_t(x.size), C.c_float(s), _p(out))
    return out


def quantize_f32(x: np.ndarray, s: float) -> np.ndarray:
    x = _f32(x)
    out = np.empty(x.shape, np.int8)
    lib().orc_quantize_f32(_p(x), C.c_size_t(x.size), C.c_float(s), _p(out))
    return out


def quantize_weight(W: np.ndarray):
    W = _f16(W)
    N, K = W.shape
    Wq = np.empty((N, K), np.int8)
    s_w = np.empty(N, np.float32)
    lib().orc_quantize_weight(_p(W), N, K, _p(Wq), _p(s_w))
    return Wq, s_w


def gemm_i8_i32(A: np.ndarray, W: np.ndarray) -> np.ndarray:
    A = np.ascontiguousarray(A, np.int8)
    W = np.ascontiguousarray(W, np.int8)
    M, K = A.shape
    N, K2 = W.shape
    assert K == K2
    out = np.empty((M, N), np.int32)
    lib().orc_gemm_i8_i32(_p(A), _p(W), _p(out), M, N, K)
    return out


def fold_requant(s_in: float, s_w: np.ndarray, bias: Optional[np.ndarray], s_out: float):
    s_w = _f32(s_w)
    N = s_w.size
    m = np.empty(N, np.float32)
    b = np.empty(N, np.float32)
    bias = None if bias is None else _f32(bias)
    lib().orc_fold_requant(C.c_float(s_in), _p(s_w), _p(bias), C.c_float(s_out), N, _p(m), _p(b))
    return m, b


def fold_dequant(s_in: float, s_w: np.ndarray) -> np.ndarray:
    s_w = _f32(s_w)
    m = np.empty(s_w.size, np.float32)
    lib().orc_fold_dequant(C.c_float(s_in), _p(s_w), s_w.size, _p(m))
    return m


def epilogue_requant(acc: np.ndarray, m: np.ndarray, b: np.ndarray) -> np.ndarray:
    acc = np.ascontiguousarray(acc, np.int32)
    M, N = acc.shape
    out = np.empty((M, N), np.int8)
    lib().orc_epilogue_requant(_p(acc), M, N, _p(_f32(m)), _p(_f32(b)), _p(out))
    return out


def epilogue_gelu_quant(acc: np.ndarray, m: np.ndarray, bias: np.ndarray, s_out: float) -> np.ndarray:
    acc = np.ascontiguousarray(acc, np.int32)
    M, N = acc.shape
    out = np.empty((M, N), np.int8)
    lib().orc_epilogue_gelu_quant(_p(acc), M, N, _p(_f32(m)), _p(_f32(bias)), C.c_float(s_out), _p(out))
    return out


def attention_i8(qkv: np.ndarray, cu: np.ndarray, heads: int, s_q, s_k, s_v, s_p, s_ctx, dump_p: bool = False,
                 p_unsigned: bool = False):
    """p_unsigned: softmax codes 0..255 with step s_p (= absmax/255) instead of the symmetric -127..127."""
    qkv = np.ascontiguousarray(qkv, np.int8)
    cu = np.ascontiguousarray(cu, np.int32)
    T, H3 = qkv.shape
    H = H3 // 3
    ctx = np.zeros((T, H), np.int8)
    pd = None
    if dump_p:
        n = int(cu[-1] - cu[-2])
        pd = np.zeros((heads, n, n), np.uint8)
    lib().orc_attention_i8(_p(qkv), _p(cu), cu.size - 1, H, heads, C.c_float(s_q), C.c_float(s_k), C.c_float(s_v),
                           C.c_float(s_p), C.c_float(s_ctx), int(bool(p_unsigned)), _p(ctx), _p(pd))
    if dump_p and not p_unsigned:
        pd = pd.view(np.int8)
    return (ctx, pd) if dump_p else ctx


def attention_i8_p16(qkv: np.ndarray, cu: np.ndarray, heads: int, s_q, s_k, s_v, s_ctx) -> np.ndarray:
    """INT8 attention block whose softmax output stays in binary16 (no step s_p): int8 context [T, H]."""
    qkv = np.ascontiguousarray(qkv, np.int8)
    cu = np.ascontiguousarray(cu, np.int32)
    T, H3 = qkv.shape
    H = H3 // 3
    ctx = np.zeros((T, H), np.int8)
    lib().orc_attention_i8_p16(_p(qkv), _p(cu), cu.size - 1, H, heads, C.c_float(s_q), C.c_float(s_k), C.c_float(s_v),
                               C.c_float(s_ctx), _p(ctx))
    return ctx


def attention_f16(qkv: np.ndarray, cu: np.ndarray, heads: int) -> np.ndarray:
    qkv = _f16(qkv)
    cu = np.ascontiguousarray(cu, np.int32)
    T, H3 = qkv.shape
    H = H3 // 3
    ctx = np.zeros((T, H), np.float16)
    lib().orc_attention_f16(_p(qkv), _p(cu), cu.size - 1, H, heads, _p(ctx))
    return ctx


def gemm_f16(A: np.ndarray, W: np.ndarray, bias: Optional[np.ndarray], gelu_flag: bool) -> np.ndarray:
    A = _f16(A)
    W = _f16(W)
    M, K = A.shape
    N, K2 = W.shape
    assert K == K2
    out = np.empty((M, N), np.float16)
    bias = None if bias is None else _f32(bias)
    lib().orc_gemm_f16(_p(A), _p(W), _p(bias), int(gelu_flag), _p(out), M, N, K)
    return out


def add_ln(inp: np.ndarray, s_in: float, bias: np.ndarray, res: np.ndarray, s_res: float,
           gamma: np.ndarray, beta: np.ndarray, eps: float, out_i8: bool, s_out: float = 1.0) -> np.ndarray:
    """Fused dequant + bias + residual + LayerNorm (+ quant).  int8 arrays are codes with the given step."""
    inp = np.ascontiguousarray(inp)
    res = np.ascontiguousarray(res)
    M, H = inp.shape
    in_i8 = inp.dtype == np.int8
    res_i8 = res.dtype == np.int8
    assert in_i8 or inp.dtype == np.float16
    assert res_i8 or res.dtype == np.float16
    out = np.empty((M, H), np.int8 if out_i8 else np.float16)
    lib().orc_add_ln(_p(inp), int(in_i8), C.c_float(s_in), _p(_f32(bias)), _p(res), int(res_i8), C.c_float(s_res),
                     _p(_f32(gamma)), _p(_f32(beta)), C.c_float(eps), _p(out), int(out_i8), C.c_float(s_out), M, H)
    return out


class _Embedding(C.Structure):
    _fields_ = [("tok", C.c_void_p), ("seg", C.c_void_p), ("pos", C.c_void_p), ("gamma", C.c_void_p), ("beta", C.c_void_p),
                ("vocab", C.c_int32), ("segments", C.c_int32), ("positions", C.c_int32), ("eps", C.c_float)]


def _embedding(emb: Dict[str, np.ndarray]):
    """emb: tok [V,H], seg [G,H], pos [P,H] fp16; gamma, beta [H] fp32; eps."""
    keep = [_f16(emb["tok"]), _f16(emb["seg"]), _f16(emb["pos"]), _f32(emb["gamma"]), _f32(emb["beta"])]
    e = _Embedding(*[a.ctypes.data for a in keep], keep[0].shape[0], keep[1].shape[0], keep[2].shape[0], float(emb["eps"]))
    return e, keep


def embed_ln(emb: Dict[str, np.ndarray], token_ids: np.ndarray, segment_ids: Optional[np.ndarray], out_i8: bool,
             s_out: float = 1.0) -> np.ndarray:
    """Embedding kernel for ONE sequence: LayerNorm(tok[id] + seg[sid] + pos[s]) as fp16 or int8 codes."""
    e, keep = _embedding(emb)
    ids = np.ascontiguousarray(token_ids, np.int32)
    seg = None if segment_ids is None else np.ascontiguousarray(segment_ids, np.int32)
    H = keep[0].shape[1]
    out = np.empty((ids.size, H), np.int8 if out_i8 else np.float16)
    lib().orc_embed_ln(C.byref(e), _p(ids), _p(seg), ids.size, H, _p(out), int(out_i8), C.c_float(s_out))
    return out


# ---------------------------------------------------------------- encoder
def _weights_array(weights: Sequence[Dict[str, np.ndarray]]):
    keep = []
    arr = (_LayerWeights * len(weights))()
    for i, w in enumerate(weights):
        for n in _WFIELDS:
            a = _f16(w[n]) if n.startswith("w_") else _f32(w[n])
            keep.append(a)
            setattr(arr[i], n, a.ctypes.data)
    return arr, keep


def _scales_array(scales: Optional[np.ndarray], layers: int):
    arr = (_LayerScales * layers)()
    if scales is None:
        for i in range(layers):
            for n in SCALE_FIELDS:
                setattr(arr[i], n, 1.0)
        return arr
    scales = np.asarray(scales, np.float32).reshape(layers, len(SCALE_FIELDS))
    for i in range(layers):
        for j, n in enumerate(SCALE_FIELDS):
            setattr(arr[i], n, float(scales[i, j]))
    return arr


def _config(layers, hidden, heads, ffn, ln_eps):
    return _Config(layers, hidden, heads, ffn, ln_eps)


class Encoder:
    """The mixed-precision encoder of Section 3.2 on the CPU.  modes[l]: bit0 = MHA INT8, bit1 = FFN INT8; with bit0, bit2 = unsigned
    softmax codes or bit3 = binary16 softmax output."""

    def __init__(self, layers, hidden, heads, ffn, ln_eps, modes, weights, scales):
        self.cfg = _config(layers, hidden, heads, ffn, ln_eps)
        self.hidden = hidden
        self.ffn = ffn
        self.modes = np.ascontiguousarray(modes, np.uint8)
        assert self.modes.size == layers
        warr, self._keep = _weights_array(weights)
        sarr = _scales_array(scales, layers)
        self._h = C.c_void_p(lib().orc_encoder_create(C.byref(self.cfg), _p(self.modes), warr, sarr))

    def forward(self, hidden: np.ndarray, lens: np.ndarray, nthreads: int = 0, tap_layer: Optional[int] = None):
        hidden = _f16(hidden)
        B, S, H = hidden.shape
        assert H == self.hidden
        lens = np.ascontiguousarray(lens, np.int32)
        out = np.empty((B, S, H), np.float16)
        taps_obj = None
        tapped = None
        if tap_layer is not None:
            n = int(lens[0])
            mode = int(self.modes[tap_layer])
            mha8, ffn8 = bool(mode & 1), bool(mode & 2)
            last = tap_layer == self.modes.size - 1
            next8 = (not last) and bool(self.modes[tap_layer + 1] & 1)
            dt = lambda q: np.int8 if q else np.float16
            tapped = {
                "x": np.zeros((n, H), dt(mha8)), "qkv": np.zeros((n, 3 * H), dt(mha8)),
                "ctx": np.zeros((n, H), dt(mha8)), "attn_out": np.zeros((n, H), dt(mha8)),
                "h1": np.zeros((n, H), dt(ffn8)), "ffn_mid": np.zeros((n, self.ffn), dt(ffn8)),
                "ffn_out": np.zeros((n, H), dt(ffn8)), "y": np.zeros((n, H), dt(next8)),
            }
            taps_obj = _Taps()
            taps_obj.layer = tap_layer
            for k, v in tapped.items():
                setattr(taps_obj, k, v.ctypes.data)
        rc = lib().orc_encoder_forward(self._h, _p(hidden), _p(lens), B, S, _p(out), nthreads,
                                       C.byref(taps_obj) if taps_obj is not None else None)
        if rc != 0:
            raise ValueError("oracle: sequence length outside [1, S]")
        return (out, tapped) if tap_layer is not None else out

    def forward_ids(self, emb: Dict[str, np.ndarray], token_ids: np.ndarray, segment_ids: Optional[np.ndarray],
                    lens: np.ndarray, nthreads: int = 0) -> np.ndarray:
        """The encoder with the Embedding kernel in front (ids int32 [B,S])."""
        e, keep = _embedding(emb)
        ids = np.ascontiguousarray(token_ids, np.int32)
        seg = None if segment_ids is None else np.ascontiguousarray(segment_ids, np.int32)
        B, S = ids.shape
        lens = np.ascontiguousarray(lens, np.int32)
        out = np.empty((B, S, self.hidden), np.float16)
        rc = lib().orc_encoder_forward_ids(self._h, C.byref(e), _p(ids), _p(seg), _p(lens), B, S, _p(out), nthreads)
        if rc != 0:
            raise ValueError("oracle: sequence length outside [1, S]")
        return out

    def close(self):
        if self._h:
            lib().orc_encoder_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def reference_forward(layers, hidden_size, heads, ffn, ln_eps, weights, hidden, lens, want_out=True,
                      want_absmax=False, nthreads: int = 0):
    """Unquantised binary64 forward.  Returns (out float64 [B,S,H] or None, absmax float32 [layers,10] or None)."""
    cfg = _config(layers, hidden_size, heads, ffn, ln_eps)
    warr, keep = _weights_array(weights)
    hidden = _f16(hidden)
    B, S, H = hidden.shape
    lens = np.ascontiguousarray(lens, np.int32)
    out = np.empty((B, S, H), np.float64) if want_out else None
    am = np.zeros((layers, len(SCALE_FIELDS)), np.float32) if want_absmax else None
    rc = lib().orc_reference_forward(C.byref(cfg), warr, _p(hidden), _p(lens), B, S, _p(out), _p(am), nthreads)
    if rc != 0:
        raise ValueError("oracle: sequence length outside [1, S]")
    return out, am


def calibrate(layers, hidden_size, heads, ffn, ln_eps, weights, calib_hidden, nthreads: int = 0) -> np.ndarray:
    """Min-max calibration: scales float32 [layers, 10] = absmax / 127 over the calibration batch."""
    B, S, _ = calib_hidden.shape
    lens = np.full(B, S, np.int32)
    _, am = reference_forward(layers, hidden_size, heads, ffn, ln_eps, weights, calib_hidden, lens,
                              want_out=False, want_absmax=True, nthreads=nthreads)
    sc = np.empty_like(am)
    lib().orc_scales_from_absmax(_p(am), am.size, _p(sc))
    return sc


# ---------------------------------------------------------------- downstream target
def classify(hidden: np.ndarray, w_pool: np.ndarray, b_pool: np.ndarray, w_cls: np.ndarray, b_cls: np.ndarray) -> np.ndarray:
    """Classification target on the first token (Section 3.1, "Downstream Target"; the paper's tasks are BERT text
    classification): pooled = tanh(W_p h[:, 0] + b_p), logits = W_c pooled + b_c, all in binary64.
    hidden fp16 [B,S,H]; w_pool fp16 [H,H], w_cls fp16 [C,H] (rows = outputs); biases fp32.  Returns float64 [B,C]."""
    h = np.asarray(hidden[:, 0, :], np.float64)
    pooled = np.tanh(h @ np.asarray(w_pool, np.float64).T + np.asarray(b_pool, np.float64))
    return pooled @ np.asarray(w_cls, np.float64).T + np.asarray(b_cls, np.float64)
