// Shared device helpers and the internal launcher interface of libsamp (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include <hip/hip_ext.h>
#include <stdint.h>

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

// ---- GELU -------------------------------------------------------------------------------------
// 1 + erf(u) for binary32 u through the five-term rational/exponential approximation of
// Abramowitz & Stegun 7.1.26 (|error| <= 1.5e-7 in exact arithmetic), arranged as erfc on the
// negative side so that no cancellation occurs there.
__device__ __forceinline__ float one_plus_erf_fast(float u)
{
    const float au = __builtin_fabsf(u);
    const float t = __builtin_amdgcn_rcpf(__builtin_fmaf(0.3275911f, au, 1.0f));
    float p = 1.061405429f;
    p = __builtin_fmaf(p, t, -1.453152027f);
    p = __builtin_fmaf(p, t, 1.421413741f);
    p = __builtin_fmaf(p, t, -0.284496736f);
    p = __builtin_fmaf(p, t, 0.254829592f);
    p = p * t;
    const float ex = __builtin_amdgcn_exp2f(-au * au * 1.44269504088896341f);
    const float tail = p * ex;                            // erfc(|u|)
    return u < 0.0f ? tail : 2.0f - tail;
}

__device__ __forceinline__ float gelu_fast(float y)
{
    return 0.5f * y * one_plus_erf_fast(y * 0.70710678118654752440f);
}

// GELU evaluated in binary64 and rounded once: the value the quantiser's decision is defined on.
__device__ __forceinline__ float gelu_exact(float y)
{
    const double yd = (double)y;
    const double g = 0.5 * yd * (1.0 + erf(yd * 0.70710678118654752440));
    return (float)g;
}

// Bound on |gelu_fast(y) - GELU(y)|, validated exhaustively by the GPU tests.
#define SAMP_GELU_FAST_ABS_ERR_PER_UNIT 8.0e-7f

// code = rne(GELU(y) * inv_s) from the fast GELU, plus a flag telling whether the value lies within
// the fast path's error bound of a rounding tie (then the binary64 definition has to decide).
__device__ __forceinline__ int gelu_quant_code_fast(float y, float inv_s, bool &near_tie)
{
    const float c = gelu_fast(y) * inv_s;
    const float r = __builtin_rintf(c);
    const float dist = __builtin_fabsf(__builtin_fabsf(c - r) - 0.5f);   // distance to the nearest tie
    const float margin = __builtin_fabsf(y) * inv_s * SAMP_GELU_FAST_ABS_ERR_PER_UNIT
                       + __builtin_fabsf(c) * 6.0e-7f + 1.0e-30f;
    near_tie = dist <= margin;
    return (int)__builtin_fminf(__builtin_fmaxf(r, -127.0f), 127.0f);
}

// The same decision for one value on its own.
__device__ __forceinline__ int gelu_quant_code(float y, float inv_s)
{
    bool near_tie;
    const int c = gelu_quant_code_fast(y, inv_s, near_tie);
    return near_tie ? qcode(gelu_exact(y) * inv_s) : c;
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

enum GemmEpilogue { EPI_RAW_I32, EPI_REQUANT, EPI_GELU_QUANT };
extern int gemm_config_override;                           // < 0: choose the tile configuration by shape

hipError_t launch_gemm_i8(GemmEpilogue epi, const int8_t *A, const int8_t *W, void *out, const float *m, const float *b,
                          float inv_s_out, Rows rows, int N, int K, hipStream_t st, const Timing *tm);
hipError_t launch_gemm_f16(const __half *A, const __half *W, const float *bias, bool gelu, __half *out, Rows rows,
                           int N, int K, hipStream_t st, const Timing *tm);

// cu == nullptr: every sequence has exactly max_len rows (row b*max_len is its first).
hipError_t launch_attention_i8(const int8_t *qkv, const int *cu, int B, int max_len, int H, int heads, float m_sc,
                               float inv_sp, float m_ctx, int8_t *ctx, hipStream_t st, const Timing *tm);
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

}  // namespace samp
