"""The C-ABI library loads without a GPU, exports every symbol the header declares, and turns
invalid arguments into error codes on the host (no kernel is launched here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "samp.h")


@pytest.fixture(scope="module")
def L():
    import paper_2209_09130_amd as P
    from paper_2209_09130_amd import build as B
    if not os.path.exists(P.lib_path()):
        B.build(force=True)
    return P.lib()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"SAMP_API[^;(]*?\b(samp_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = declared_symbols()
    for must in ("samp_encoder_create", "samp_encoder_forward", "samp_encoder_workspace_bytes",
                 "samp_encoder_destroy", "samp_last_error"):
        assert must in names
    assert len(names) >= 15


def test_library_exports_every_declared_symbol(L):
    for name in declared_symbols():
        assert hasattr(L, name), name


def test_invalid_arguments_become_error_codes_on_the_host(L):
    from paper_2209_09130_amd.binding import _Config
    L.samp_encoder_arena_bytes.restype = C.c_size_t
    modes = (C.c_uint8 * 2)(3, 0)
    ok = _Config(2, 768, 12, 3072, 8, 128, 1e-12)
    assert L.samp_encoder_arena_bytes(C.byref(ok), modes) > 2 * (768 * 768 * 4 + 2 * 768 * 3072)
    bad_head = _Config(2, 768, 8, 3072, 8, 128, 1e-12)
    assert L.samp_encoder_arena_bytes(C.byref(bad_head), modes) == 0
    assert b"head size" in L.samp_last_error()
    long_seq = _Config(2, 768, 12, 3072, 8, 4096, 1e-12)
    assert L.samp_encoder_arena_bytes(C.byref(long_seq), modes) > 0
    bad_seq = _Config(2, 768, 12, 3072, 8, 4097, 1e-12)
    assert L.samp_encoder_arena_bytes(C.byref(bad_seq), modes) == 0
    assert b"max_seq" in L.samp_last_error()
    too_many = _Config(2, 768, 12, 3072, 8192, 4096, 1e-12)                         # 2^25 token rows
    assert L.samp_encoder_arena_bytes(C.byref(too_many), modes) == 0
    assert b"tokens" in L.samp_last_error()
    too_wide = _Config(2, 768, 12, 3072, 8193, 16, 1e-12)                           # the sequence-offset kernel's limit
    assert L.samp_encoder_arena_bytes(C.byref(too_wide), modes) == 0
    assert b"max_batch" in L.samp_last_error()
    assert L.samp_encoder_arena_bytes(C.byref(ok), (C.c_uint8 * 2)(16, 0)) == 0
    assert L.samp_encoder_arena_bytes(C.byref(ok), (C.c_uint8 * 2)(8, 0)) == 0       # a binary16 softmax output needs an INT8 MHA
    assert L.samp_encoder_arena_bytes(C.byref(ok), (C.c_uint8 * 2)(13, 0)) == 0      # ... and excludes the unsigned codes
    assert L.samp_encoder_arena_bytes(C.byref(ok), (C.c_uint8 * 2)(9, 11)) > 0
    assert L.samp_encoder_arena_bytes(C.byref(ok), (C.c_uint8 * 2)(6, 0)) == 0       # unsigned softmax codes need an INT8 MHA
    assert L.samp_encoder_arena_bytes(C.byref(ok), (C.c_uint8 * 2)(7, 5)) > 0
    assert L.samp_encoder_arena_bytes(None, modes) == 0
    # step entry points reject NULL pointers and unsupported shapes before touching the device
    assert L.samp_gemm_i8_i32(None, None, None, 1, 128, 64, None) == -1
    buf = (C.c_char * 64)()
    assert L.samp_gemm_i8_i32(buf, buf, buf, 1, 100, 64, None) == -2
    assert L.samp_gemm_i8_i32(buf, buf, buf, 1, 128, 60, None) == -2
    assert L.samp_add_ln(None, 0, C.c_float(1), None, None, 0, C.c_float(1), None, None, C.c_float(0), None, 0,
                         C.c_float(1), 1, 768, None) == -1
    assert L.samp_encoder_workspace_bytes(None, 1, 1) == 0
    assert L.samp_encoder_destroy(None) == 0
    out = C.c_void_p()
    assert L.samp_encoder_create(C.byref(ok), modes, None, None, None, C.c_size_t(0), None, C.byref(out)) == -1
    assert L.samp_encoder_forward(None, None, None, 1, 1, None, None, C.c_size_t(0), None) == -1


def test_later_entry_points_reject_bad_arguments_on_the_host(L):
    """The embedding, target, histogram and tuning entry points check their arguments before any launch."""
    from paper_2209_09130_amd.binding import _EmbeddingStruct
    buf = (C.c_char * 256)()
    emb = _EmbeddingStruct()                                   # all pointers NULL
    assert L.samp_embed_ln(C.byref(emb), buf, None, 1, 4, 128, buf, 0, C.c_float(1), None) == -1
    assert b"NULL" in L.samp_last_error()
    assert L.samp_embed_ln(None, buf, None, 1, 4, 128, buf, 0, C.c_float(1), None) == -1
    assert L.samp_embed_ln(C.byref(emb), None, None, 1, 4, 128, buf, 0, C.c_float(1), None) == -1
    assert L.samp_encoder_forward_ids(None, C.byref(emb), buf, None, None, 1, 4, buf, buf, C.c_size_t(256), None) == -1
    assert L.samp_classify(None, 1, 4, 128, buf, buf, buf, buf, 3, buf, None) == -1
    assert L.samp_classify(buf, 1, 4, 100, buf, buf, buf, buf, 3, buf, None) == -2          # H % 8
    assert L.samp_classify(buf, 1, 4, 128, buf, buf, buf, buf, 0, buf, None) == -2          # no classes
    assert L.samp_code_histogram(None, C.c_size_t(16), buf, None) == -1
    assert L.samp_code_histogram(buf, C.c_size_t(0), buf, None) == -2
    assert L.samp_set_gemm_config(9) == -1
    assert L.samp_set_gemm_config(-1) == 0
    assert L.samp_attention_i8(None, None, 1, 16, 128, 2, C.c_float(1), C.c_float(1), C.c_float(1), C.c_float(1), C.c_float(1),
                               0, None, None, None) == -1
    assert L.samp_probe_feed_rate(buf, C.c_size_t(256), 100, 128, 128, 1, buf, None, C.byref(C.c_double())) == -2
    assert L.samp_probe_feed_rate(buf, C.c_size_t(256), 128, 128, 128, 1, buf, None, C.byref(C.c_double())) == -3   # buffer too small
    # a score multiplier s_q s_k / 8 above 256 is refused on the host (the softmax exponential's argument range)
    aligned = (C.c_char * 4096)()
    base = (C.addressof(aligned) + 255) & ~255
    ptr, cu = C.c_void_p(base), C.c_void_p(base + 2048)
    assert L.samp_attention_i8(ptr, cu, 1, 16, 128, 2, C.c_float(64), C.c_float(64), C.c_float(1), C.c_float(1), C.c_float(1),
                               0, ptr, None, None) == -5
    assert b"256" in L.samp_last_error()
    # the kernel that does the QKV GEMM and the attention at once: sequences of at most 128 tokens, head size 64
    f1 = C.c_float(0.02)
    assert L.samp_qkv_attention_i8(None, ptr, ptr, None, cu, 1, 16, 128, 2, f1, f1, f1, f1, f1, 0, ptr, None) == -1
    assert L.samp_qkv_attention_i8(ptr, ptr, ptr, None, cu, 1, 257, 128, 2, f1, f1, f1, f1, f1, 0, ptr, None) == -2
    assert L.samp_qkv_attention_i8(ptr, ptr, ptr, None, cu, 1, 16, 100, 2, f1, f1, f1, f1, f1, 0, ptr, None) == -2
    assert L.samp_qkv_attention_i8(ptr, ptr, ptr, None, cu, 1, 16, 128, 2, f1, f1, f1, f1, f1, 2, ptr, None) == -1   # no binary16 softmax output here
    assert L.samp_qkv_attention_i8(ptr, ptr, ptr, None, cu, 1, 16, 128, 2, C.c_float(64), C.c_float(64), f1, f1, f1, 0, ptr, None) == -5
    assert L.samp_encoder_set_qkv_fusion(None, 0) == -1
    assert L.samp_qkv_attention_f16(ptr, ptr, None, cu, 1, 257, 128, 2, ptr, None) == -2
    assert L.samp_qkv_attention_f16(ptr, None, None, cu, 1, 16, 128, 2, ptr, None) == -1
