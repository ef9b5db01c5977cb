// Shared device helpers and the internal launcher interface of libsamp (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_ext.h>
#include <stdint.h>

#include <atomic>

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v16i __attribute__((ext_vector_type(16)));
typedef float v4f __attribute__((ext_vector_type(4)));
typedef float v16f __attribute__((ext_vector_type(16)));
typedef _Float16 v8h __attribute__((ext_vector_type(8)));
typedef _Float16 v4h __attribute__((ext_vector_type(4)));

namespace samp {

// ---- quantiser: round half to even, symmetric clamp (Appendix B) --------------------------------
__device__ __forceinline__ int qcode(float v)
{
    float r = __builtin_rintf(v);                        // v_rndne_f32
    r = __builtin_fminf(__builtin_fmaxf(r, -127.0f), 127.0f);
    return (int)r;
}

// binary32 -> binary16 as a separate, single rounding step.  The empty asm keeps the compiler from
// folding a preceding multiply-add into a mixed-precision FMA that rounds to binary16 directly,
// which would skip the binary32 rounding the results are defined with.
__device__ __forceinline__ _Float16 to_half(float v)
{
    asm("" : "+v"(v));
    return (_Float16)v;
}

__device__ __forceinline__ int pack4(int a, int b, int c, int d)
{
    return (a & 0xff) | ((b & 0xff) << 8) | ((c & 0xff) << 16) | ((unsigned)(d & 0xff) << 24);
}

// The quantiser without integer conversions.  Clamping before rounding gives the same code as
// clamping after it (the bounds are integers), and adding 1.5 * 2^23 to a value of magnitude below
// 2^22 rounds it to an integer, ties to even, in the adder itself; the sum's bit pattern then holds
// the code in two's complement in its low byte.  code_bits() returns that pattern, pack_codes()
// gathers the low bytes of four of them into one dword with byte permutes.
#define SAMP_RNE_MAGIC 12582912.0f
__device__ __forceinline__ float code_bits(float v)
{
    return __builtin_amdgcn_fmed3f(v, -127.0f, 127.0f) + SAMP_RNE_MAGIC;
}
__device__ __forceinline__ int pack_codes(float f0, float f1, float f2, float f3)
{
    const unsigned lo = __builtin_amdgcn_perm(__float_as_uint(f1), __float_as_uint(f0), 0x0c0c0400u);
    const unsigned hi = __builtin_amdgcn_perm(__float_as_uint(f3), __float_as_uint(f2), 0x0c0c0400u);
    return (int)__builtin_amdgcn_perm(hi, lo, 0x05040100u);
}
__device__ __forceinline__ int code_of_bits(float f) { return (int)(int8_t)(__float_as_uint(f) & 0xffu); }

// ---- GELU -------------------------------------------------------------------------------------
// erfc(|u|) / 2 at u = y / sqrt(2) through the five-term rational/exponential approximation of
// Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7 on erfc in exact arithmetic).  The argument is
// pre-scaled by sqrt(log2 e) so that the exponential is a bare exp2 of -(v*v), and the halving is
// folded into the polynomial's coefficients.
__device__ __forceinline__ float half_erfc_fast(float y)
{
    const float v = y * 0.84932180028801904f;              // y / sqrt(2) * sqrt(log2 e)
    const float ex = __builtin_amdgcn_exp2f(-(v * v));
    const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.27273748087922248f, __builtin_fabsf(v), 1.0f));
    float p = 0.5307027145f;
    p = __builtin_fmaf(p, t, -0.7265760135f);
    p = __builtin_fmaf(p, t, 0.7107068705f);
    p = __builtin_fmaf(p, t, -0.142248368f);
    p = __builtin_fmaf(p, t, 0.127414796f);
    return (p * t) * ex;
}

// k * GELU(y) from yk = k * y (k > 0), as relu(yk) - |yk| * erfc(|u|)/2: no cancellation on either
// side of zero, and the scale rides along for free.
__device__ __forceinline__ float gelu_scaled_fast(float y, float yk)
{
    return __builtin_fmaf(-__builtin_fabsf(yk), half_erfc_fast(y), __builtin_fmaxf(yk, 0.0f));
}

__device__ __forceinline__ float gelu_fast(float y) { return gelu_scaled_fast(y, y); }

// GELU evaluated in binary64 and rounded once: the value the quantiser's decision is defined on.
__device__ __forceinline__ float gelu_exact(float y)
{
    const double yd = (double)y;
    const double g = 0.5 * yd * (1.0 + erf(yd * 0.70710678118654752440));
    return (float)g;
}

// Bound on |gelu_fast(y) - GELU(y)| per unit of |y|, validated by a dense sweep in the GPU tests; the
// tie test below adds 6e-7 per unit for the binary32 roundings on either side of the comparison.
#define SAMP_GELU_FAST_ABS_ERR_PER_UNIT 8.0e-7f
#define SAMP_GELU_TIE_MARGIN_PER_UNIT (SAMP_GELU_FAST_ABS_ERR_PER_UNIT + 6.0e-7f)

// code_bits of rne(GELU(y) * inv_s) from the fast GELU, plus a flag telling whether the scaled value
// lies within the fast path's error bound of a rounding tie (then the binary64 definition decides).
// |GELU(y)| <= |y|, so |y| * inv_s bounds both error terms.
__device__ __forceinline__ float gelu_code_bits_fast(float y, float inv_s, bool &near_tie)
{
    const float yk = y * inv_s;
    const float c = __builtin_amdgcn_fmed3f(gelu_scaled_fast(y, yk), -127.0f, 127.0f);
    const float f = c + SAMP_RNE_MAGIC;
    const float d = c - (f - SAMP_RNE_MAGIC);
    near_tie = __builtin_fabsf(__builtin_fabsf(d) - 0.5f) <= __builtin_fabsf(yk) * SAMP_GELU_TIE_MARGIN_PER_UNIT;
    return f;
}

// The same decision for one value on its own.
__device__ __forceinline__ int gelu_quant_code(float y, float inv_s)
{
    bool near_tie;
    const float f = gelu_code_bits_fast(y, inv_s, near_tie);
    return near_tie ? qcode(gelu_exact(y) * inv_s) : code_of_bits(f);
}

// ---- work-group -> work-item mapping that keeps tokens on one XCD --------------------------------
// The hardware hands consecutive work-groups of a dispatch to the 8 XCDs in turn, and each XCD has its
// own L2: what one kernel leaves in an XCD's L2 is a hit for the next kernel only if the block that
// reads it runs on the same XCD (measured: handing 6 MB from kernel to kernel costs 2.5 us per link
// when producer and consumer blocks share the XCD, 5.2 us when they do not).  Every kernel of the
// path therefore numbers its work items (row tiles, row blocks, sequences) so that XCD x owns the
// x-th eighth of them, i.e. the same eighth of the token rows in every kernel.  The last total % 8
// items keep their own index.
__device__ __forceinline__ int xcd_contiguous(int block, int total)
{
    const int per = total >> 3, body = per << 3;
    return block < body ? (block & 7) * per + (block >> 3) : block;
}

// ---- wave reductions (64 lanes) ----------------------------------------------------------------
__device__ __forceinline__ double wave_sum(double v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}
__device__ __forceinline__ float wave_max(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = __builtin_fmaxf(v, __shfl_xor(v, o, 64));
    return v;
}

// ---- host-side launcher interface (implemented in the .hip files) -------------------------------
struct Timing { hipEvent_t start, stop; };                 // optional events attached to one dispatch

// Plain launch, or (tm != nullptr) a launch whose dispatch carries start/stop events.  Event-carrying
// dispatches cannot be captured into a graph, so they are only used when timing was asked for.
template <class K, class... Args>
inline void launch_kernel(K kern, dim3 grid, dim3 block, size_t lds, hipStream_t st, const Timing *tm, Args... args)
{
    if (tm) hipExtLaunchKernelGGL(kern, grid, block, lds, st, tm->start, tm->stop, 0, args...);
    else hipLaunchKernelGGL(kern, grid, block, lds, st, args...);
}

// Row limit of a launch: rows = *dev_rows if dev_rows != nullptr, else host_rows.
struct Rows { int host_rows; const int *dev_rows; };

// Threshold table of the FFN1 epilogue (gelu_table.hip): bin(y) = low mantissa bits of
// med3(fmaf(y, rate, offset), 2^23, t_max); entry i = { binary32 Y_i, lo | hi << 8 }, code = y >= Y_i ? hi : lo.
constexpr int GELU_TABLE_MAX_BINS = 2048;
struct GeluTableSpec { float rate, offset, t_max; int bins; };
bool gelu_table_build(float inv_s, GeluTableSpec *sp, uint32_t *entries /* host, 2 * GELU_TABLE_MAX_BINS */);
struct GeluTable { GeluTableSpec spec; const uint32_t *entries; };        // entries: device memory, 2 * spec.bins words

enum GemmEpilogue { EPI_RAW_I32, EPI_REQUANT, EPI_GELU_QUANT };
extern std::atomic<int> gemm_config_override;                           // < 0: choose the tile configuration by shape

// gelu_table (EPI_GELU_QUANT only, may be null): the threshold table of this inv_s_out; without it the epilogue
// evaluates GELU per element (certified binary32 fast path, binary64 where a rounding tie is near)
hipError_t launch_gemm_i8(GemmEpilogue epi, const int8_t *A, const int8_t *W, void *out, const float *m, const float *b,
                          float inv_s_out, const GeluTable *gelu_table, Rows rows, int N, int K, hipStream_t st,
                          const Timing *tm);
hipError_t launch_gemm_f16(const __half *A, const __half *W, const float *bias, bool gelu, __half *out, Rows rows,
                           int N, int K, hipStream_t st, const Timing *tm);

// cu == nullptr: every sequence has exactly max_len rows (row b*max_len is its first).
// p_unsigned: softmax codes 0..255 instead of -127..127; p_hist (optional): 256 counters of the codes used
hipError_t launch_attention_i8(const int8_t *qkv, const int *cu, int B, int max_len, int H, int heads, float m_sc,
                               float inv_sp, float m_ctx, bool p_unsigned, int8_t *ctx, unsigned long long *p_hist,
                               hipStream_t st, const Timing *tm);
hipError_t launch_qkv_attention_i8(const int8_t *x, const int8_t *w_qkv, const float *m, const float *b, const int *cu, int B,
                                   int max_len, int H, float m_sc, float inv_sp, float m_ctx, bool p_unsigned, int8_t *ctx,
                                   hipStream_t st, const Timing *tm);
hipError_t launch_qkv_attention_f16(const __half *x, const __half *w_qkv, const float *bias, const int *cu, int B, int max_len,
                                    int H, float scale, __half *ctx, hipStream_t st, const Timing *tm);
hipError_t launch_code_histogram(const int8_t *codes, size_t n, unsigned long long *hist, hipStream_t st);
hipError_t launch_attention_i8_p16(const int8_t *qkv, const int *cu, int B, int max_len, int H, int heads, float m_sc,
                                   float m_ctx, int8_t *ctx, hipStream_t st, const Timing *tm);
hipError_t launch_attention_f16(const __half *qkv, const int *cu, int B, int max_len, int H, int heads, float scale,
                                __half *ctx, float *p_absmax, hipStream_t st, const Timing *tm);

struct AddLnArgs {
    const void *in; bool in_i8; float s_in; const float *bias;
    const void *res; bool res_i8; float s_res;
    const float *gamma, *beta; float eps;
    void *out; bool out_i8; float s_out;
    const int *row_map;                                    // optional: output row of packed row t
    float *absmax_out;                                     // optional: running absmax of y (calibration)
    Rows rows; int H;
};
hipError_t launch_add_ln(const AddLnArgs &a, hipStream_t st, const Timing *tm);

struct EmbedArgs {
    const int *token_ids, *segment_ids;                    // [B*S]; segment_ids may be null (segment 0)
    const __half *tok, *seg, *pos; int vocab, segments, positions;
    const float *gamma, *beta; float eps;
    const int *cu;                                         // null: every sequence has S rows and row b*S+s is written
    int B, S, H;
    void *out; bool out_i8; float s_out;
    int *row_map;                                          // with cu: output row of packed row t
    __half *out_zero_pad;                                  // with cu: [B*S, H] whose padded rows are zeroed
};
hipError_t launch_embed_ln(const EmbedArgs &a, hipStream_t st, const Timing *tm);

hipError_t launch_quantize_weight(const __half *W, int N, int K, int8_t *Wq, float *s_w, hipStream_t st);
hipError_t launch_fold(const float *s_in_dev_or_null, float s_in, const float *s_w, const float *bias, float s_out, int N,
                       float *m, float *b, hipStream_t st);
hipError_t launch_seq_offsets(const int *mask, int B, int S, int *cu, hipStream_t st);
hipError_t launch_pack_rows(const __half *hidden, const int *cu, int B, int S, int H, float s_x, void *packed,
                            int *row_map, __half *out_zero_pad, hipStream_t st, const Timing *tm);
hipError_t launch_quantize_rows(const __half *x, size_t n, float s_x, int8_t *out, hipStream_t st, const Timing *tm);
hipError_t launch_absmax_f16(const __half *x, Rows rows, int cols, int ld, float *slot, hipStream_t st);
hipError_t launch_fill_f32(float *p, int n, float v, hipStream_t st);
hipError_t launch_gelu_quant(const float *y, size_t n, float inv_s, int8_t *codes, float *fast, hipStream_t st);

hipError_t launch_classify(const __half *hidden, int B, int S, int H, const __half *w_pool, const float *b_pool,
                           const __half *w_cls, const float *b_cls, int C, float *logits, hipStream_t st);

// measured ceilings (probe.hip); both synchronise the stream
hipError_t probe_mfma_rate(bool f16, bool random_operands, int iters, int *sink, hipStream_t st, double *ops_per_s);
hipError_t probe_copy_rate(const void *src, void *dst, size_t bytes, int reps, hipStream_t st, double *bytes_per_s);
hipError_t probe_feed_rate(const void *A, const void *W, int rows, int N, int kbytes, int reps, int *sink, hipStream_t st,
                           double *bytes_per_s);

// host-side recommendation logic (allocator.hip)
int allocate_decay_aware(const double *A, const double *L, int n);
int recommend_settings(const double *A, const double *L, int n, double max_latency, double min_accuracy, int *out, int cap);

}  // namespace samp
