"""ctypes binding of the C ABI in include/samp.h (same names, argument marshalling only)."""
from __future__ import annotations

import ctypes as C
import os
from typing import List, Dict, Optional, Sequence

import numpy as np
import torch

FP16, MHA_INT8, FFN_INT8, FULL_INT8 = 0, 1, 2, 3
P_UNSIGNED = 4
P_FP16 = 8
(PROF_OFF, PROF_QKV, PROF_ATTN, PROF_ATTN_OUT, PROF_LN1, PROF_FFN1, PROF_FFN2, PROF_LN2, PROF_ENTRY, PROF_QKV_ATTN) = range(10)
SCALE_FIELDS = ("x", "q", "k", "v", "p", "ctx", "attn_out", "ffn_in", "ffn_mid", "ffn_out")

_PKG = os.path.dirname(os.path.abspath(__file__))


class SampError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"libsamp error {code}: {msg}")
        self.code = code


class _Config(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("layers", "hidden", "heads", "ffn", "max_batch", "max_seq")] + \
               [("ln_eps", C.c_float)]


_WFIELDS = ("w_qkv", "w_o", "w_ffn1", "w_ffn2", "b_qkv", "b_o", "b_ffn1", "b_ffn2",
            "ln1_g", "ln1_b", "ln2_g", "ln2_b")


class _LayerWeights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in _WFIELDS]


class _LayerScales(C.Structure):
    _fields_ = [(n, C.c_float) for n in SCALE_FIELDS]


def lib_path() -> str:
    return os.path.join(_PKG, "libsamp.so")


_lib = None


def lib():
    """Loads libsamp.so.  There is no fallback: without the HIP library nothing here works."""
    global _lib
    if _lib is None:
        path = lib_path()
        if not os.path.exists(path):
            raise ImportError(f"{path} is missing: build it first (python -m paper_2209_09130_amd.build)")
        L = C.CDLL(path)
        L.samp_last_error.restype = C.c_char_p
        L.samp_encoder_arena_bytes.restype = C.c_size_t
        L.samp_encoder_workspace_bytes.restype = C.c_size_t
        L.samp_encoder_workspace_bytes.argtypes = [C.c_void_p, C.c_int32, C.c_int32]
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        raise SampError(rc, lib().samp_last_error().decode())


def _stream() -> C.c_void_p:
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _dp(t: Optional[torch.Tensor]) -> C.c_void_p:
    if t is None:
        return C.c_void_p(0)
    assert t.is_cuda and t.is_contiguous()
    return C.c_void_p(t.data_ptr())


def _f(v) -> C.c_float:
    return C.c_float(float(v))


class _EmbeddingStruct(C.Structure):
    _fields_ = [("token_table", C.c_void_p), ("segment_table", C.c_void_p), ("position_table", C.c_void_p),
                ("gamma", C.c_void_p), ("beta", C.c_void_p), ("vocab", C.c_int32), ("segments", C.c_int32),
                ("positions", C.c_int32), ("ln_eps", C.c_float)]


class Embedding:
    """Device copies of the embedding tables and the samp_embedding_t that points at them."""

    def __init__(self, tok: np.ndarray, seg: np.ndarray, pos: np.ndarray, gamma: np.ndarray, beta: np.ndarray, eps: float):
        assert tok.dtype == seg.dtype == pos.dtype == np.float16
        self.tok, self.seg, self.pos = (torch.from_numpy(np.ascontiguousarray(a)).cuda() for a in (tok, seg, pos))
        self.gamma, self.beta = (torch.from_numpy(np.ascontiguousarray(a, np.float32)).cuda() for a in (gamma, beta))
        self.hidden = tok.shape[1]
        self.struct = _EmbeddingStruct()            # ctypes zero-fills, padding included
        self.struct.token_table, self.struct.segment_table, self.struct.position_table = (
            self.tok.data_ptr(), self.seg.data_ptr(), self.pos.data_ptr())
        self.struct.gamma, self.struct.beta = self.gamma.data_ptr(), self.beta.data_ptr()
        self.struct.vocab, self.struct.segments, self.struct.positions = tok.shape[0], seg.shape[0], pos.shape[0]
        self.struct.ln_eps = float(eps)


def embed_ln(emb: Embedding, token_ids: torch.Tensor, segment_ids: Optional[torch.Tensor], out_i8: bool,
             s_out: float = 1.0) -> torch.Tensor:
    """samp_embed_ln: [B*S, H] fp16 or int8 codes."""
    assert token_ids.dtype == torch.int32 and token_ids.dim() == 2
    B, S = token_ids.shape
    out = torch.zeros((B * S, emb.hidden), dtype=torch.int8 if out_i8 else torch.float16, device=token_ids.device)
    _check(lib().samp_embed_ln(C.byref(emb.struct), _dp(token_ids), _dp(segment_ids), B, S, emb.hidden, _dp(out),
                               int(bool(out_i8)), _f(s_out), _stream()))
    return out


class Encoder:
    """samp_encoder_create / forward / calibrate / destroy."""

    def __init__(self, layers: int, hidden: int, heads: int, ffn: int, ln_eps: float, modes: Sequence[int],
                 weights: Sequence[Dict[str, np.ndarray]], scales: Optional[np.ndarray], max_batch: int, max_seq: int,
                 device: str = "cuda:0"):
        L = lib()
        self.device = torch.device(device)
        torch.cuda.set_device(self.device)
        self.cfg = _Config(layers, hidden, heads, ffn, max_batch, max_seq, ln_eps)
        self.layers, self.hidden = layers, hidden
        modes_arr = (C.c_uint8 * layers)(*[int(m) for m in modes])
        keep = []
        warr = (_LayerWeights * layers)()
        for i, w in enumerate(weights):
            for n in _WFIELDS:
                a = np.ascontiguousarray(w[n], dtype=np.float16 if n.startswith("w_") else np.float32)
                keep.append(a)
                setattr(warr[i], n, a.ctypes.data)
        sarr = None
        if scales is not None:
            sc = np.asarray(scales, np.float32).reshape(layers, len(SCALE_FIELDS))
            sarr = (_LayerScales * layers)()
            for i in range(layers):
                for j, n in enumerate(SCALE_FIELDS):
                    setattr(sarr[i], n, float(sc[i, j]))
        nbytes = L.samp_encoder_arena_bytes(C.byref(self.cfg), modes_arr)
        if nbytes == 0:
            raise SampError(-1, L.samp_last_error().decode())
        self.arena = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
        self._h = C.c_void_p()
        _check(L.samp_encoder_create(C.byref(self.cfg), modes_arr, warr, sarr, _dp(self.arena), C.c_size_t(nbytes),
                                     _stream(), C.byref(self._h)))
        self._ws = None

    def workspace_bytes(self, B: int, S: int) -> int:
        return int(lib().samp_encoder_workspace_bytes(self._h, B, S))

    def _workspace(self, B: int, S: int) -> torch.Tensor:
        need = self.workspace_bytes(B, S)
        if need == 0:
            raise SampError(-1, lib().samp_last_error().decode())
        if self._ws is None or self._ws.numel() < need:
            self._ws = torch.empty(need, dtype=torch.uint8, device=self.device)
        return self._ws

    def forward(self, hidden: torch.Tensor, mask: Optional[torch.Tensor] = None,
                out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """samp_encoder_forward.  Pass the same `out` tensor on every call to get graph replay: the library keys its
        recorded graphs on the argument pointers, and a fresh output tensor per call is a new argument set each time
        (plain launches, and it pushes older graphs out of the cache)."""
        assert hidden.dtype == torch.float16 and hidden.dim() == 3
        B, S, H = hidden.shape
        ws = self._workspace(B, S)
        if out is None:
            out = torch.empty_like(hidden)
        if mask is not None:
            assert mask.dtype == torch.int32 and tuple(mask.shape) == (B, S)
        _check(lib().samp_encoder_forward(self._h, _dp(hidden), _dp(mask), B, S, _dp(out), _dp(ws),
                                          C.c_size_t(ws.numel()), _stream()))
        return out

    def forward_noalloc(self, hidden: torch.Tensor, mask: Optional[torch.Tensor], out: torch.Tensor) -> torch.Tensor:
        """samp_encoder_forward_noalloc: the workspace is the library's built-in scratch array; nothing is allocated."""
        assert hidden.dtype == torch.float16 and hidden.dim() == 3 and out.shape == hidden.shape and out.dtype == torch.float16
        B, S, H = hidden.shape
        if mask is not None:
            assert mask.dtype == torch.int32 and tuple(mask.shape) == (B, S)
        _check(lib().samp_encoder_forward_noalloc(self._h, _dp(hidden), _dp(mask), B, S, _dp(out), _stream()))
        return out

    def forward_ids(self, emb: "Embedding", token_ids: torch.Tensor, segment_ids: Optional[torch.Tensor] = None,
                    mask: Optional[torch.Tensor] = None, out: Optional[torch.Tensor] = None) -> torch.Tensor:
        """samp_encoder_forward_ids: the Embedding kernel feeds layer 0 directly."""
        assert token_ids.dtype == torch.int32 and token_ids.dim() == 2
        B, S = token_ids.shape
        ws = self._workspace(B, S)
        if out is None:
            out = torch.empty((B, S, emb.hidden), dtype=torch.float16, device=token_ids.device)
        _check(lib().samp_encoder_forward_ids(self._h, C.byref(emb.struct), _dp(token_ids), _dp(segment_ids), _dp(mask),
                                              B, S, _dp(out), _dp(ws), C.c_size_t(ws.numel()), _stream()))
        return out

    def calibrate(self, hidden: torch.Tensor, mask: Optional[torch.Tensor] = None) -> np.ndarray:
        B, S, H = hidden.shape
        ws = self._workspace(B, S)
        out = (_LayerScales * self.layers)()
        _check(lib().samp_encoder_calibrate(self._h, _dp(hidden), _dp(mask), B, S, _dp(ws), C.c_size_t(ws.numel()),
                                            _stream(), out))
        return np.array([[getattr(out[i], n) for n in SCALE_FIELDS] for i in range(self.layers)], np.float32)

    def set_groups(self, groups: int):
        _check(lib().samp_encoder_set_groups(self._h, int(groups)))

    def set_qkv_fusion(self, mode: int):
        """0: QKV GEMM + attention in one kernel where it is faster, 1: never, 2: whenever the shape allows."""
        _check(lib().samp_encoder_set_qkv_fusion(self._h, int(mode)))

    def set_graph(self, enabled: bool):
        _check(lib().samp_encoder_set_graph(self._h, int(bool(enabled))))

    def profile(self, which: int):
        _check(lib().samp_encoder_profile(self._h, int(which)))

    def profile_read(self):
        ms, n = C.c_double(), C.c_int64()
        _check(lib().samp_encoder_profile_read(self._h, C.byref(ms), C.byref(n)))
        return ms.value, n.value

    def close(self):
        if getattr(self, "_h", None) is not None and self._h:
            lib().samp_encoder_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


# ---- single steps (same names as the C entry points without the samp_ prefix) ----------------------
def gemm_i8_i32(A: torch.Tensor, W: torch.Tensor) -> torch.Tensor:
    M, K = A.shape
    N = W.shape[0]
    out = torch.empty((M, N), dtype=torch.int32, device=A.device)
    _check(lib().samp_gemm_i8_i32(_dp(A), _dp(W), _dp(out), M, N, K, _stream()))
    return out


def gemm_i8_requant(A, W, m, b) -> torch.Tensor:
    M, K = A.shape
    N = W.shape[0]
    out = torch.empty((M, N), dtype=torch.int8, device=A.device)
    _check(lib().samp_gemm_i8_requant(_dp(A), _dp(W), _dp(m), _dp(b), _dp(out), M, N, K, _stream()))
    return out


class _GeluTable(C.Structure):
    _fields_ = [("rate", C.c_float), ("offset", C.c_float), ("t_max", C.c_float), ("bins", C.c_int32)]


def gelu_table_build(s_out: float):
    """samp_gelu_table_build: (description struct, host entries uint32 [bins, 2]) of the FFN1 epilogue's table."""
    buf = np.zeros(4096, np.uint32)
    spec = _GeluTable()
    _check(lib().samp_gelu_table_build(_f(s_out), C.byref(spec), buf.ctypes.data_as(C.c_void_p), C.c_size_t(buf.nbytes)))
    return spec, buf[: 2 * spec.bins].reshape(spec.bins, 2).copy()


def gemm_i8_gelu_quant(A, W, m, bias, s_out: float, table=None) -> torch.Tensor:
    """table: None for the per-element evaluation, or (description, device entries) from gelu_table_build(s_out)."""
    M, K = A.shape
    N = W.shape[0]
    out = torch.empty((M, N), dtype=torch.int8, device=A.device)
    spec, entries = (None, None) if table is None else table
    _check(lib().samp_gemm_i8_gelu_quant(_dp(A), _dp(W), _dp(m), _dp(bias), _f(s_out),
                                         C.byref(spec) if spec is not None else None, _dp(entries), _dp(out), M, N, K, _stream()))
    return out


def gemm_f16(A, W, bias, gelu: bool) -> torch.Tensor:
    M, K = A.shape
    N = W.shape[0]
    out = torch.empty((M, N), dtype=torch.float16, device=A.device)
    _check(lib().samp_gemm_f16(_dp(A), _dp(W), _dp(bias), int(gelu), _dp(out), M, N, K, _stream()))
    return out


def _batch_of(cu, T: int, max_len: int) -> int:
    if cu is not None:
        return cu.numel() - 1
    assert T % max_len == 0, "without sequence offsets every sequence has max_len rows"
    return T // max_len


def attention_i8(qkv, cu, max_len: int, heads: int, s_q, s_k, s_v, s_p, s_ctx, p_unsigned: bool = False,
                 want_hist: bool = False, p_fp16: bool = False):
    """Returns ctx, or (ctx, hist) with hist = int64 [256] counts of the softmax codes (index = code byte).
    p_fp16: the softmax output stays binary16 (s_p unused, no histogram).
    cu None: qkv holds T / max_len sequences of exactly max_len rows each."""
    assert not (p_fp16 and (p_unsigned or want_hist))
    T, H3 = qkv.shape
    H = H3 // 3
    B = _batch_of(cu, T, max_len)
    ctx = torch.zeros((T, H), dtype=torch.int8, device=qkv.device)
    hist = torch.zeros(256, dtype=torch.int64, device=qkv.device) if want_hist else None
    _check(lib().samp_attention_i8(_dp(qkv), _dp(cu), B, max_len, H, heads, _f(s_q), _f(s_k), _f(s_v),
                                   _f(s_p), _f(s_ctx), 2 if p_fp16 else int(bool(p_unsigned)), _dp(ctx), _dp(hist), _stream()))
    return (ctx, hist) if want_hist else ctx


def qkv_attention_i8(x, w_qkv, m, b, cu, max_len: int, heads: int, s_q, s_k, s_v, s_p, s_ctx, p_unsigned: bool = False):
    """samp_qkv_attention_i8: ctx [T, H] int8 from packed int8 rows x [T, H] and the int8 QKV weights [3H, H]."""
    T, H = x.shape
    B = _batch_of(cu, T, max_len)
    ctx = torch.zeros((T, H), dtype=torch.int8, device=x.device)
    _check(lib().samp_qkv_attention_i8(_dp(x), _dp(w_qkv), _dp(m), _dp(b), _dp(cu), B, max_len, H, heads, _f(s_q), _f(s_k),
                                       _f(s_v), _f(s_p), _f(s_ctx), int(bool(p_unsigned)), _dp(ctx), _stream()))
    return ctx


def qkv_attention_f16(x, w_qkv, bias, cu, max_len: int, heads: int):
    """samp_qkv_attention_f16: ctx [T, H] fp16 from packed fp16 rows x [T, H] and the fp16 QKV weights [3H, H]."""
    T, H = x.shape
    B = _batch_of(cu, T, max_len)
    ctx = torch.zeros((T, H), dtype=torch.float16, device=x.device)
    _check(lib().samp_qkv_attention_f16(_dp(x), _dp(w_qkv), _dp(bias), _dp(cu), B, max_len, H, heads, _dp(ctx), _stream()))
    return ctx


def classify(hidden: torch.Tensor, w_pool, b_pool, w_cls, b_cls) -> torch.Tensor:
    """samp_classify: float32 logits [B, classes] from the first token of each sequence."""
    B, S, H = hidden.shape
    Cn = w_cls.shape[0]
    logits = torch.zeros((B, Cn), dtype=torch.float32, device=hidden.device)
    _check(lib().samp_classify(_dp(hidden), B, S, H, _dp(w_pool), _dp(b_pool), _dp(w_cls), _dp(b_cls), Cn, _dp(logits), _stream()))
    return logits


def code_histogram(codes: torch.Tensor) -> torch.Tensor:
    """int64 [256] counts of an int8 tensor's byte values (index = the code as an unsigned byte)."""
    assert codes.dtype == torch.int8
    hist = torch.zeros(256, dtype=torch.int64, device=codes.device)
    _check(lib().samp_code_histogram(_dp(codes), C.c_size_t(codes.numel()), _dp(hist), _stream()))
    return hist


def attention_f16(qkv, cu, max_len: int, heads: int) -> torch.Tensor:
    T, H3 = qkv.shape
    H = H3 // 3
    ctx = torch.zeros((T, H), dtype=torch.float16, device=qkv.device)
    _check(lib().samp_attention_f16(_dp(qkv), _dp(cu), _batch_of(cu, T, max_len), max_len, H, heads, _dp(ctx), _stream()))
    return ctx


def add_ln(inp, s_in, bias, res, s_res, gamma, beta, eps, out_i8: bool, s_out: float = 1.0) -> torch.Tensor:
    M, H = inp.shape
    out = torch.empty((M, H), dtype=torch.int8 if out_i8 else torch.float16, device=inp.device)
    _check(lib().samp_add_ln(_dp(inp), int(inp.dtype == torch.int8), _f(s_in), _dp(bias), _dp(res),
                             int(res.dtype == torch.int8), _f(s_res), _dp(gamma), _dp(beta), _f(eps), _dp(out),
                             int(out_i8), _f(s_out), M, H, _stream()))
    return out


def gelu_quant(y: torch.Tensor, s_out: float, want_fast: bool = False):
    n = y.numel()
    codes = torch.empty(n, dtype=torch.int8, device=y.device)
    fast = torch.empty(n, dtype=torch.float32, device=y.device) if want_fast else None
    _check(lib().samp_gelu_quant(_dp(y), C.c_int64(n), _f(s_out), _dp(codes), _dp(fast), _stream()))
    return (codes, fast) if want_fast else codes


def quantize_f16_i8(x: torch.Tensor, s_x: float) -> torch.Tensor:
    """samp_quantize_f16_i8: int8 codes of an fp16 tensor (element count a multiple of 8)."""
    assert x.dtype == torch.float16
    out = torch.empty(x.shape, dtype=torch.int8, device=x.device)
    _check(lib().samp_quantize_f16_i8(_dp(x), C.c_int64(x.numel()), _f(s_x), _dp(out), _stream()))
    return out


def quantize_weight(W: torch.Tensor):
    N, K = W.shape
    Wq = torch.empty((N, K), dtype=torch.int8, device=W.device)
    s_w = torch.empty(N, dtype=torch.float32, device=W.device)
    _check(lib().samp_quantize_weight(_dp(W), N, K, _dp(Wq), _dp(s_w), _stream()))
    return Wq, s_w


def allocate_decay_aware(accuracy: Sequence[float], latency: Sequence[float]) -> int:
    """samp_allocate_decay_aware: index of the setting Algorithm 1 recommends."""
    n = len(accuracy)
    assert n == len(latency)
    a = (C.c_double * n)(*[float(v) for v in accuracy])
    l = (C.c_double * n)(*[float(v) for v in latency])
    out = C.c_int32(-1)
    _check(lib().samp_allocate_decay_aware(a, l, n, C.byref(out)))
    return int(out.value)


def recommend(accuracy: Sequence[float], latency: Sequence[float], max_latency: Optional[float] = None,
              min_accuracy: Optional[float] = None) -> List[int]:
    """samp_recommend: the Appendix A rules; thresholds left None are unset."""
    n = len(accuracy)
    assert n == len(latency)
    a = (C.c_double * n)(*[float(v) for v in accuracy])
    l = (C.c_double * n)(*[float(v) for v in latency])
    out = (C.c_int32 * 8)()
    cnt = C.c_int32(0)
    nan = float("nan")
    _check(lib().samp_recommend(a, l, n, C.c_double(nan if max_latency is None else max_latency),
                                C.c_double(nan if min_accuracy is None else min_accuracy), out, 8, C.byref(cnt)))
    return [int(out[i]) for i in range(cnt.value)]


def set_gemm_config(config: int) -> None:
    """Force a GEMM tile configuration (0, 1, 2) or -1 to choose by shape again."""
    _check(lib().samp_set_gemm_config(int(config)))


def pack_rows(hidden: torch.Tensor, mask: torch.Tensor, s_x: float = 0.0):
    """Returns (packed [B*S,H] (first T rows valid), cu_seqlens [B+1], row_map [B*S])."""
    B, S, H = hidden.shape
    packed = torch.zeros((B * S, H), dtype=torch.int8 if s_x > 0 else torch.float16, device=hidden.device)
    cu = torch.zeros(B + 1, dtype=torch.int32, device=hidden.device)
    row_map = torch.zeros(B * S, dtype=torch.int32, device=hidden.device)
    _check(lib().samp_pack_rows(_dp(hidden), _dp(mask), B, S, H, _f(s_x), _dp(packed), _dp(cu), _dp(row_map), _stream()))
    return packed, cu, row_map


def probe_mfma_rate(fp16: bool, random_operands: bool, iters: int = 20000) -> float:
    """samp_probe_mfma_rate: measured operations per second of the matrix instruction (2 per multiply-add)."""
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = C.c_double(0.0)
    _check(lib().samp_probe_mfma_rate(int(fp16), int(random_operands), int(iters), _dp(sink), _stream(), C.byref(out)))
    return out.value


def probe_feed_rate(rows: int, N: int, kbytes: int, reps: int = 20) -> float:
    """samp_probe_feed_rate: bytes per second the blocks of a rows x N GEMM pull into LDS with no arithmetic."""
    nbytes = (rows + N) * kbytes
    buf = torch.ones(nbytes, dtype=torch.uint8, device="cuda")
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    out = C.c_double(0.0)
    _check(lib().samp_probe_feed_rate(_dp(buf), C.c_size_t(nbytes), int(rows), int(N), int(kbytes), int(reps), _dp(sink),
                                      _stream(), C.byref(out)))
    return out.value


def probe_copy_rate(nbytes: int = 1 << 30, reps: int = 10) -> float:
    """samp_probe_copy_rate: measured bytes per second (read + written) of a device copy."""
    src = torch.ones(nbytes, dtype=torch.uint8, device="cuda")
    dst = torch.empty_like(src)
    out = C.c_double(0.0)
    _check(lib().samp_probe_copy_rate(_dp(src), _dp(dst), C.c_size_t(nbytes), int(reps), _stream(), C.byref(out)))
    return out.value
