"""MI355X (gfx950) self-adaptive mixed-precision encoder: Python binding of libsamp.so.

The binding only marshals arguments; every step of the path runs in the HIP kernels behind the
C ABI declared in include/samp.h.  PyTorch is used for device memory and streams.
"""
from .binding import (  # noqa: F401
    Encoder, Embedding, embed_ln, SampError, lib, lib_path,
    FP16, MHA_INT8, FFN_INT8, FULL_INT8, P_UNSIGNED, P_FP16, SCALE_FIELDS,
    PROF_OFF, PROF_QKV, PROF_ATTN, PROF_ATTN_OUT, PROF_LN1, PROF_FFN1, PROF_FFN2, PROF_LN2, PROF_ENTRY, PROF_QKV_ATTN,
    gemm_i8_i32, gemm_i8_requant, gemm_i8_gelu_quant, gelu_table_build, gemm_f16, attention_i8, qkv_attention_i8, qkv_attention_f16, attention_f16, add_ln,
    quantize_weight, quantize_f16_i8, pack_rows, gelu_quant, set_gemm_config, allocate_decay_aware, recommend, code_histogram, classify, probe_mfma_rate, probe_copy_rate, probe_feed_rate,
)
