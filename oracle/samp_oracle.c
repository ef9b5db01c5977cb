/*
 * CPU oracle of the self-adaptive mixed-precision encoder (SAMP, arXiv 2209.09130).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, step-by-step statement of
 * what the encoder hot path computes, used only to check the HIP library and to
 * time a CPU baseline.  It shares no code with the HIP path and nothing in the
 * product may call it.
 *
 * What the paper fixes (Section 3.2, Section 4.2, Appendix B):
 *   - every layer's attention block (MHA) and feed-forward block (FFN) runs
 *     either in floating point or with INT8 GEMMs ("Fully-Quant" = both INT8,
 *     "Quant-FFN-Only" = FFN INT8 with a float MHA);
 *   - post-training quantisation with scales fixed by a min-max calibration:
 *     multiply by a scale, round to an integer, symmetric 8-bit range;
 *   - in a quantised block every tensor that travels between kernels is int8;
 *     dequantise + bias + residual + LayerNorm + quantise form one step; the
 *     softmax output is quantised too; the last step of a layer whose consumer
 *     is floating point does not quantise.
 * What it leaves open (rounding mode, clamp, where biases enter, which scales
 * exist, GELU form) is read as stated at each function below.
 *
 * Precision rules used throughout:
 *   - integer accumulations are exact int32;
 *   - every value that decides an int8 code is formed by a fixed sequence of
 *     IEEE binary32 operations (explicit fmaf / single multiplies) so that an
 *     implementation with fp32 epilogues can take the same decision;
 *   - reductions (LayerNorm statistics, softmax denominators, fp16 GEMM dot
 *     products) and transcendentals (exp, erf) are evaluated in binary64 and
 *     rounded once to binary32;
 *   - binary16 conversion is round-to-nearest-even, written out below.
 * Compile with -ffp-contract=off so that no multiply-add is fused silently.
 *
 * Parity pins: see tests/test_oracle_*.py.  The absolute values of a full
 * quantised layer have no worked example in the paper: beyond the invariants
 * and brute-force checks there, they are "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORC_API __attribute__((visibility("default")))

enum { ORC_MHA_INT8 = 1, ORC_FFN_INT8 = 2,
       ORC_P_UNSIGNED = 4,     /* with ORC_MHA_INT8: softmax codes 0..255 instead of the symmetric range */
       ORC_P_FP16 = 8 };       /* with ORC_MHA_INT8, not with ORC_P_UNSIGNED: the softmax output stays binary16 */

/* ------------------------------------------------------------------------ */
/* binary16 <-> binary32 (IEEE 754, round to nearest even)                   */
/* ------------------------------------------------------------------------ */
static inline uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static inline float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

static float h2f(uint16_t h)
{
    uint32_t sign = (uint32_t)(h & 0x8000u) << 16;
    uint32_t e = (h >> 10) & 0x1fu, m = h & 0x3ffu;
    if (e == 0) {                       /* zero or subnormal: m * 2^-24, exact in binary32 */
        float v = (float)m * 0x1p-24f;
        return sign ? -v : v;
    }
    if (e == 31) return bits_f32(sign | 0x7f800000u | (m << 13));
    return bits_f32(sign | ((e + 112u) << 23) | (m << 13));
}

static uint16_t f2h(float f)
{
    uint32_t x = f32_bits(f);
    uint16_t sign = (uint16_t)((x >> 16) & 0x8000u);
    x &= 0x7fffffffu;
    if (x > 0x7f800000u) return (uint16_t)(sign | 0x7e00u);        /* NaN */
    if (x >= 0x477ff000u) return (uint16_t)(sign | 0x7c00u);       /* >= 65520 rounds to inf */
    if (x < 0x38800000u) {                                         /* below 2^-14: subnormal half */
        float scaled = bits_f32(x) * 0x1p24f;                      /* exact power-of-two scaling */
        uint32_t m = (uint32_t)nearbyintf(scaled);                 /* RNE; 1024 becomes the least normal */
        return (uint16_t)(sign | m);
    }
    uint32_t e = (x >> 23) - 112u, mant = x & 0x7fffffu;
    uint32_t half = (e << 10) | (mant >> 13), rem = mant & 0x1fffu;
    if (rem > 0x1000u || (rem == 0x1000u && (half & 1u))) half++;  /* carry may bump the exponent */
    return (uint16_t)(sign | half);
}

ORC_API void orc_f16_to_f32(const uint16_t *in, float *out, size_t n)
{ for (size_t i = 0; i < n; i++) out[i] = h2f(in[i]); }

ORC_API void orc_f32_to_f16(const float *in, uint16_t *out, size_t n)
{ for (size_t i = 0; i < n; i++) out[i] = f2h(in[i]); }

/* ------------------------------------------------------------------------ */
/* Quantiser (Appendix B: scale, round, symmetric 8-bit range)               */
/* Reading: round-half-to-even, clamp to [-127, 127], scale = absmax / 127.  */
/* ------------------------------------------------------------------------ */
static inline int8_t qcode(float v)
{
    float r = nearbyintf(v);            /* default rounding mode = nearest even */
    if (!(r == r)) r = 0.0f;            /* NaN is an input error; keep it defined */
    if (r > 127.0f) r = 127.0f;
    if (r < -127.0f) r = -127.0f;
    return (int8_t)r;
}

ORC_API int orc_quant_code(float v) { return qcode(v); }

/* quantise fp16 activations with a per-tensor step s: code = rne(x * (1/s)) */
ORC_API void orc_quantize_f16(const uint16_t *x, size_t n, float s, int8_t *out)
{
    float inv_s = 1.0f / s;
    for (size_t i = 0; i < n; i++) out[i] = qcode(h2f(x[i]) * inv_s);
}

ORC_API void orc_quantize_f32(const float *x, size_t n, float s, int8_t *out)
{
    float inv_s = 1.0f / s;
    for (size_t i = 0; i < n; i++) out[i] = qcode(x[i] * inv_s);
}

/* Weights (Section 4.1: scales "convert model weights from floating-point to
 * fixed-point").  Reading: one step per output channel (row of W[out,in]),
 * s_w = absmax / 127 (1 if the row is all zero), code = rne(w / s_w).        */
ORC_API void orc_quantize_weight(const uint16_t *W, int N, int K, int8_t *Wq, float *s_w)
{
    for (int n = 0; n < N; n++) {
        float amax = 0.0f;
        for (int k = 0; k < K; k++) { float a = fabsf(h2f(W[(size_t)n * K + k])); if (a > amax) amax = a; }
        float s = amax > 0.0f ? amax / 127.0f : 1.0f;
        s_w[n] = s;
        for (int k = 0; k < K; k++) Wq[(size_t)n * K + k] = qcode(h2f(W[(size_t)n * K + k]) / s);
    }
}

/* ------------------------------------------------------------------------ */
/* INT8 GEMM: acc[t,n] = sum_k A[t,k] * W[n,k], exact int32                   */
/* ------------------------------------------------------------------------ */
static int8_t *transpose_i8(const int8_t *W, int N, int K)
{
    int8_t *Wt = (int8_t *)malloc((size_t)N * K);
    for (int n = 0; n < N; n++) for (int k = 0; k < K; k++) Wt[(size_t)k * N + n] = W[(size_t)n * K + k];
    return Wt;
}

/* Wt is W stored [K][N]; the k-loop order per output is the natural 0..K-1 */
static void gemm_i8_t(const int8_t *A, const int8_t *Wt, int32_t *C, int M, int N, int K)
{
    for (int t = 0; t < M; t++) {
        int32_t *c = C + (size_t)t * N;
        for (int n = 0; n < N; n++) c[n] = 0;
        for (int k = 0; k < K; k++) {
            int32_t a = A[(size_t)t * K + k];
            const int8_t *w = Wt + (size_t)k * N;
            for (int n = 0; n < N; n++) c[n] += a * (int32_t)w[n];
        }
    }
}

ORC_API void orc_gemm_i8_i32(const int8_t *A, const int8_t *W, int32_t *C, int M, int N, int K)
{
    int8_t *Wt = transpose_i8(W, N, K);
    gemm_i8_t(A, Wt, C, M, N, K);
    free(Wt);
}

/* ------------------------------------------------------------------------ */
/* Epilogue tables.  A multiplier that combines several steps is formed in    */
/* binary64 from the binary32 steps and rounded once.                         */
/* ------------------------------------------------------------------------ */
/* requantising epilogue: code = rne(fmaf(acc, m[n], b[n]))
 *   m[n] = s_in * s_w[n] / s_out,  b[n] = bias[n] / s_out (0 if bias == NULL) */
ORC_API void orc_fold_requant(float s_in, const float *s_w, const float *bias, float s_out, int N, float *m, float *b)
{
    for (int n = 0; n < N; n++) {
        m[n] = (float)((double)s_in * (double)s_w[n] / (double)s_out);
        b[n] = bias ? (float)((double)bias[n] / (double)s_out) : 0.0f;
    }
}

/* dequantising multiplier: m[n] = s_in * s_w[n] (real units) */
ORC_API void orc_fold_dequant(float s_in, const float *s_w, int N, float *m)
{
    for (int n = 0; n < N; n++) m[n] = (float)((double)s_in * (double)s_w[n]);
}

ORC_API void orc_epilogue_requant(const int32_t *acc, int M, int N, const float *m, const float *b, int8_t *out)
{
    for (int t = 0; t < M; t++)
        for (int n = 0; n < N; n++)
            out[(size_t)t * N + n] = qcode(fmaf((float)acc[(size_t)t * N + n], m[n], b[n]));
}

/* GELU in its exact form 0.5 x (1 + erf(x / sqrt 2)) (the paper's models are
 * BERT; the form is the reading), evaluated in binary64, rounded to binary32 */
static inline float gelu_f32(float y)
{
    double yd = (double)y;
    double g = 0.5 * yd * (1.0 + erf(yd * 0.70710678118654752440));
    return (float)g;
}
ORC_API float orc_gelu(float y) { return gelu_f32(y); }

/* FFN1 epilogue: y = fmaf(acc, m[n], bias[n]) in real units, g = GELU(y),
 * code = rne(g * (1/s_out)) */
ORC_API void orc_epilogue_gelu_quant(const int32_t *acc, int M, int N, const float *m, const float *bias,
                                     float s_out, int8_t *out)
{
    float inv_s = 1.0f / s_out;
    for (int t = 0; t < M; t++)
        for (int n = 0; n < N; n++) {
            float y = fmaf((float)acc[(size_t)t * N + n], m[n], bias[n]);
            out[(size_t)t * N + n] = qcode(gelu_f32(y) * inv_s);
        }
}

/* ------------------------------------------------------------------------ */
/* Softmax row shared by both attention flavours.                             */
/* sc[0..n) -> e[j] = fl32(exp(sc[j] - max)), S = fl32(sum e in binary64),     */
/* returns rS = 1/S; the normalised value is P[j] = e[j] * rS.                */
/* ------------------------------------------------------------------------ */
static float softmax_row(const float *sc, int n, float *e)
{
    float mx = sc[0];
    for (int j = 1; j < n; j++) if (sc[j] > mx) mx = sc[j];
    double S = 0.0;
    for (int j = 0; j < n; j++) { e[j] = (float)exp((double)(sc[j] - mx)); S += (double)e[j]; }
    return 1.0f / (float)S;
}

/* INT8 attention (Section 4.2 / Appendix B: the softmax output is quantised,
 * so both batched products are int8 x int8 -> int32).
 * qkv: int8 [T, 3H], columns [0,H) = Q, [H,2H) = K, [2H,3H) = V; head h owns
 * columns h*d .. h*d+d-1 of each third.  cu: sequence b owns rows cu[b]..cu[b+1).
 * Only the keys of the same sequence take part (padding is never stored).
 *   score = fl32(acc) * m_sc,        m_sc  = s_q * s_k / sqrt(d)
 *   Pq    = rne(P * (1/s_p))   clamped to [-127, 127]  (p_unsigned == 0: the
 *           symmetric code of Appendix B, whose negative half a softmax output
 *           never uses) or to [0, 255] (p_unsigned != 0: the variant Section 4.2
 *           points to, spending all 256 codes on [0, 1]; s_p is then absmax/255)
 *   ctx   = rne(fl32(sum_j Pq V) * m_ctx),  m_ctx = s_p * s_v / s_ctx
 * p_dump (optional): [heads][n][n] codes of the LAST sequence, one byte each
 * (0..127 or 0..255; a softmax code is never negative).                       */
static inline int32_t pcode(float v, int p_unsigned)
{
    float r = nearbyintf(v);
    if (!(r == r)) r = 0.0f;
    float hi = p_unsigned ? 255.0f : 127.0f, lo = p_unsigned ? 0.0f : -127.0f;
    if (r > hi) r = hi;
    if (r < lo) r = lo;
    return (int32_t)r;
}

ORC_API void orc_attention_i8(const int8_t *qkv, const int32_t *cu, int B, int H, int heads,
                              float s_q, float s_k, float s_v, float s_p, float s_ctx,
                              int p_unsigned, int8_t *ctx, uint8_t *p_dump)
{
    int d = H / heads;
    float m_sc = (float)((double)s_q * (double)s_k / sqrt((double)d));
    float m_ctx = (float)((double)s_p * (double)s_v / (double)s_ctx);
    float inv_sp = 1.0f / s_p;
    for (int b = 0; b < B; b++) {
        int t0 = cu[b], n = cu[b + 1] - cu[b];
        float *sc = (float *)malloc(sizeof(float) * n), *e = (float *)malloc(sizeof(float) * n);
        int32_t *pq = (int32_t *)malloc(sizeof(int32_t) * n);
        for (int h = 0; h < heads; h++)
            for (int i = 0; i < n; i++) {
                const int8_t *q = qkv + (size_t)(t0 + i) * 3 * H + h * d;
                for (int j = 0; j < n; j++) {
                    const int8_t *k = qkv + (size_t)(t0 + j) * 3 * H + H + h * d;
                    int32_t acc = 0;
                    for (int c = 0; c < d; c++) acc += (int32_t)q[c] * (int32_t)k[c];
                    sc[j] = (float)acc * m_sc;
                }
                float rS = softmax_row(sc, n, e);
                for (int j = 0; j < n; j++) {
                    float P = e[j] * rS;
                    pq[j] = pcode(P * inv_sp, p_unsigned);
                    if (p_dump && b == B - 1) p_dump[((size_t)h * n + i) * n + j] = (uint8_t)pq[j];
                }
                for (int c = 0; c < d; c++) {
                    int32_t O = 0;
                    for (int j = 0; j < n; j++)
                        O += pq[j] * (int32_t)qkv[(size_t)(t0 + j) * 3 * H + 2 * H + h * d + c];
                    ctx[(size_t)(t0 + i) * H + h * d + c] = qcode((float)O * m_ctx);
                }
            }
        free(sc); free(e); free(pq);
    }
}

/* INT8 attention block whose softmax output is NOT put on the 8-bit grid (the
 * other way out of the problem Section 4.2 / Appendix B describe: a softmax
 * output wastes most of a symmetric int8 code): scores from integers exactly
 * as above; the normalised value is rounded to binary16 and multiplies the
 * integer V codes:
 *   P16 = fl16(e[j] * rS);  ctx = rne(fl32(sum_j P16[j] * V[j]) * m),  m = s_v / s_ctx.
 * Every P16 is an integer multiple of 2^-24 not above 1 and V an integer below
 * 2^7, so each product and every partial sum (below 2^53 * 2^-24 for any row
 * length here) is exact in binary64: fl32 rounds the true sum once.            */
ORC_API void orc_attention_i8_p16(const int8_t *qkv, const int32_t *cu, int B, int H, int heads,
                                  float s_q, float s_k, float s_v, float s_ctx, int8_t *ctx)
{
    int d = H / heads;
    float m_sc = (float)((double)s_q * (double)s_k / sqrt((double)d));
    float m = (float)((double)s_v / (double)s_ctx);
    for (int b = 0; b < B; b++) {
        int t0 = cu[b], n = cu[b + 1] - cu[b];
        float *sc = (float *)malloc(sizeof(float) * n), *e = (float *)malloc(sizeof(float) * n);
        double *p = (double *)malloc(sizeof(double) * n);
        for (int h = 0; h < heads; h++)
            for (int i = 0; i < n; i++) {
                const int8_t *q = qkv + (size_t)(t0 + i) * 3 * H + h * d;
                for (int j = 0; j < n; j++) {
                    const int8_t *k = qkv + (size_t)(t0 + j) * 3 * H + H + h * d;
                    int32_t acc = 0;
                    for (int c = 0; c < d; c++) acc += (int32_t)q[c] * (int32_t)k[c];
                    sc[j] = (float)acc * m_sc;
                }
                float rS = softmax_row(sc, n, e);
                for (int j = 0; j < n; j++) p[j] = (double)h2f(f2h(e[j] * rS));
                for (int c = 0; c < d; c++) {
                    double O = 0.0;
                    for (int j = 0; j < n; j++)
                        O += p[j] * (double)qkv[(size_t)(t0 + j) * 3 * H + 2 * H + h * d + c];
                    ctx[(size_t)(t0 + i) * H + h * d + c] = qcode((float)O * m);
                }
            }
        free(sc); free(e); free(p);
    }
}

/* FP16 attention: fp16 q,k,v; score = fl32(dot in binary64) * fl32(1/sqrt d);
 * P rounded to fp16 before P.V; context rounded to fp16.                      */
ORC_API void orc_attention_f16(const uint16_t *qkv, const int32_t *cu, int B, int H, int heads, uint16_t *ctx)
{
    int d = H / heads;
    float scale = (float)(1.0 / sqrt((double)d));
    for (int b = 0; b < B; b++) {
        int t0 = cu[b], n = cu[b + 1] - cu[b];
        float *sc = (float *)malloc(sizeof(float) * n), *e = (float *)malloc(sizeof(float) * n);
        double *p = (double *)malloc(sizeof(double) * n);
        for (int h = 0; h < heads; h++)
            for (int i = 0; i < n; i++) {
                const uint16_t *q = qkv + (size_t)(t0 + i) * 3 * H + h * d;
                for (int j = 0; j < n; j++) {
                    const uint16_t *k = qkv + (size_t)(t0 + j) * 3 * H + H + h * d;
                    double acc = 0.0;
                    for (int c = 0; c < d; c++) acc += (double)h2f(q[c]) * (double)h2f(k[c]);
                    sc[j] = (float)acc * scale;
                }
                float rS = softmax_row(sc, n, e);
                for (int j = 0; j < n; j++) p[j] = (double)h2f(f2h(e[j] * rS));
                for (int c = 0; c < d; c++) {
                    double O = 0.0;
                    for (int j = 0; j < n; j++)
                        O += p[j] * (double)h2f(qkv[(size_t)(t0 + j) * 3 * H + 2 * H + h * d + c]);
                    ctx[(size_t)(t0 + i) * H + h * d + c] = f2h((float)O);
                }
            }
        free(sc); free(e); free(p);
    }
}

/* ------------------------------------------------------------------------ */
/* FP16 GEMM: fp16 operands, dot product in binary64 rounded to binary32,     */
/* + bias (binary32 add), optional GELU, rounded to fp16.                     */
/* ------------------------------------------------------------------------ */
static float *transpose_f16_to_f32(const uint16_t *W, int N, int K)
{
    float *Wt = (float *)malloc(sizeof(float) * (size_t)N * K);
    for (int n = 0; n < N; n++) for (int k = 0; k < K; k++) Wt[(size_t)k * N + n] = h2f(W[(size_t)n * K + k]);
    return Wt;
}

static void gemm_f16_t(const uint16_t *A, const float *Wt, const float *bias, int gelu, uint16_t *out,
                       int M, int N, int K)
{
    double *acc = (double *)malloc(sizeof(double) * N);
    for (int t = 0; t < M; t++) {
        for (int n = 0; n < N; n++) acc[n] = 0.0;
        for (int k = 0; k < K; k++) {
            double a = (double)h2f(A[(size_t)t * K + k]);
            const float *w = Wt + (size_t)k * N;
            for (int n = 0; n < N; n++) acc[n] += a * (double)w[n];
        }
        for (int n = 0; n < N; n++) {
            float y = (float)acc[n];
            if (bias) y = y + bias[n];
            if (gelu) y = gelu_f32(y);
            out[(size_t)t * N + n] = f2h(y);
        }
    }
    free(acc);
}

ORC_API void orc_gemm_f16(const uint16_t *A, const uint16_t *W, const float *bias, int gelu, uint16_t *out,
                          int M, int N, int K)
{
    float *Wt = transpose_f16_to_f32(W, N, K);
    gemm_f16_t(A, Wt, bias, gelu, out, M, N, K);
    free(Wt);
}

/* ------------------------------------------------------------------------ */
/* The fused step of Section 3.2: dequantise + AddBias + AddResidual +        */
/* LayerNorm (+ quantise).                                                    */
/*   z[c]  = (in[c] (* s_in) + bias[c]) + res[c] (* s_res)                    */
/*   mu, var (biased) over the H channels in binary64; rstd = 1/sqrt(var+eps) */
/*   y[c]  = fmaf((z[c] - mu32) * rstd32, gamma[c], beta[c])                  */
/*   out   = rne(y * (1/s_out)) as int8, or y rounded to fp16                 */
/* int8 operands are dequantised inside a fused multiply-add:                 */
/*   t = fmaf(in_q, s_in, bias);  z = fmaf(res_q, s_res, t)                   */
/* fp16 operands: t = in + bias; z = t + res (binary32 adds).                 */
/* ------------------------------------------------------------------------ */
/* LayerNorm of one row z[H] and its output conversion, as described above */
static void ln_row(const float *z, int H, const float *gamma, const float *beta, float eps,
                   void *out, size_t o, int out_i8, float inv_s)
{
    double mu = 0.0, var = 0.0;
    for (int c = 0; c < H; c++) mu += (double)z[c];
    mu /= (double)H;
    for (int c = 0; c < H; c++) { double dlt = (double)z[c] - mu; var += dlt * dlt; }
    var /= (double)H;
    float mu32 = (float)mu;
    float rstd32 = (float)(1.0 / sqrt(var + (double)eps));
    for (int c = 0; c < H; c++) {
        float y = fmaf((z[c] - mu32) * rstd32, gamma[c], beta[c]);
        if (out_i8) ((int8_t *)out)[o + c] = qcode(y * inv_s);
        else ((uint16_t *)out)[o + c] = f2h(y);
    }
}

ORC_API void orc_add_ln(const void *in, int in_i8, float s_in, const float *bias,
                        const void *res, int res_i8, float s_res,
                        const float *gamma, const float *beta, float eps,
                        void *out, int out_i8, float s_out, int M, int H)
{
    float *z = (float *)malloc(sizeof(float) * H);
    float inv_s = out_i8 ? 1.0f / s_out : 0.0f;
    for (int t = 0; t < M; t++) {
        size_t o = (size_t)t * H;
        for (int c = 0; c < H; c++) {
            float a = in_i8 ? fmaf((float)((const int8_t *)in)[o + c], s_in, bias[c])
                            : h2f(((const uint16_t *)in)[o + c]) + bias[c];
            z[c] = res_i8 ? fmaf((float)((const int8_t *)res)[o + c], s_res, a)
                          : a + h2f(((const uint16_t *)res)[o + c]);
        }
        ln_row(z, H, gamma, beta, eps, out, o, out_i8, inv_s);
    }
    free(z);
}

/* ------------------------------------------------------------------------ */
/* Embedding kernel (Section 3.1, "Embedding": the token, segment and        */
/* position embeddings of BERT are summed in ONE kernel; Section 3.2: for a   */
/* quantised first block the module hands INT8 to the encoder directly).      */
/* BERT's embedding ends with a LayerNorm, which belongs to the same kernel.  */
/*   z[c] = (tok[id][c] + seg[sid][c]) + pos[s][c]    binary32 adds of fp16   */
/*   out  = LayerNorm(z) as in the fused step above: fp16, or rne(y / s_out)  */
/* The token at position s of a sequence uses pos[s].  segment_ids == NULL    */
/* means segment 0.  Ids outside their table are clamped into it.             */
/* ------------------------------------------------------------------------ */
typedef struct {
    const uint16_t *tok, *seg, *pos;    /* fp16 tables [vocab][H], [segments][H], [positions][H] */
    const float *gamma, *beta;
    int32_t vocab, segments, positions;
    float eps;
} orc_embedding;

static int clampi(int v, int hi) { return v < 0 ? 0 : (v > hi ? hi : v); }

ORC_API void orc_embed_ln(const orc_embedding *E, const int32_t *token_ids, const int32_t *segment_ids,
                          int n, int H, void *out, int out_i8, float s_out)
{
    float *z = (float *)malloc(sizeof(float) * H);
    float inv_s = out_i8 ? 1.0f / s_out : 0.0f;
    for (int s = 0; s < n; s++) {
        const uint16_t *t = E->tok + (size_t)clampi(token_ids[s], E->vocab - 1) * H;
        const uint16_t *g = E->seg + (size_t)clampi(segment_ids ? segment_ids[s] : 0, E->segments - 1) * H;
        const uint16_t *p = E->pos + (size_t)clampi(s, E->positions - 1) * H;
        for (int c = 0; c < H; c++) {
            float a = h2f(t[c]) + h2f(g[c]);
            z[c] = a + h2f(p[c]);
        }
        ln_row(z, H, E->gamma, E->beta, E->eps, out, (size_t)s * H, out_i8, inv_s);
    }
    free(z);
}

/* ------------------------------------------------------------------------ */
/* Encoder object                                                             */
/* ------------------------------------------------------------------------ */
typedef struct { int32_t layers, hidden, heads, ffn; float ln_eps; } orc_config;

typedef struct {            /* fp16 matrices [out,in] row-major; fp32 vectors */
    const uint16_t *w_qkv, *w_o, *w_ffn1, *w_ffn2;
    const float *b_qkv, *b_o, *b_ffn1, *b_ffn2, *ln1_g, *ln1_b, *ln2_g, *ln2_b;
} orc_layer_weights;

/* activation steps (absmax / 127) of one layer, in dataflow order:
 * x = block input, q k v = projections with bias, p = softmax output,
 * ctx = P.V, attn_out = W_o product before its bias, ffn_in = LayerNorm-1
 * output, ffn_mid = GELU output, ffn_out = FFN2 product before its bias      */
typedef struct { float x, q, k, v, p, ctx, attn_out, ffn_in, ffn_mid, ffn_out; } orc_layer_scales;

typedef struct {
    int mode;
    /* INT8 blocks */
    int8_t *qkv_t, *o_t, *f1_t, *f2_t;         /* transposed int8 weights [K][N] */
    float *m_qkv, *b_qkv_q, *m_o, *m_f1, *m_f2, *zero_h;
    /* FP16 blocks */
    float *qkv_f, *o_f, *f1_f, *f2_f;          /* transposed fp16 weights as float [K][N] */
    /* always */
    float *b_qkv, *b_o, *b_f1, *b_f2, *g1, *be1, *g2, *be2;
    orc_layer_scales s;
} orc_layer;

typedef struct { orc_config cfg; orc_layer *L; } orc_encoder;

static float *dupf(const float *p, int n) { float *q = (float *)malloc(sizeof(float) * n); memcpy(q, p, sizeof(float) * n); return q; }

static int8_t *quant_transposed(const uint16_t *W, int N, int K, float *s_w)
{
    int8_t *Wq = (int8_t *)malloc((size_t)N * K);
    orc_quantize_weight(W, N, K, Wq, s_w);
    int8_t *Wt = transpose_i8(Wq, N, K);
    free(Wq);
    return Wt;
}

ORC_API orc_encoder *orc_encoder_create(const orc_config *cfg, const uint8_t *modes,
                                        const orc_layer_weights *w, const orc_layer_scales *sc)
{
    int H = cfg->hidden, F = cfg->ffn;
    orc_encoder *E = (orc_encoder *)calloc(1, sizeof(orc_encoder));
    E->cfg = *cfg;
    E->L = (orc_layer *)calloc(cfg->layers, sizeof(orc_layer));
    for (int l = 0; l < cfg->layers; l++) {
        orc_layer *Y = &E->L[l];
        Y->mode = modes[l];
        Y->s = sc[l];
        Y->b_qkv = dupf(w[l].b_qkv, 3 * H); Y->b_o = dupf(w[l].b_o, H);
        Y->b_f1 = dupf(w[l].b_ffn1, F);     Y->b_f2 = dupf(w[l].b_ffn2, H);
        Y->g1 = dupf(w[l].ln1_g, H); Y->be1 = dupf(w[l].ln1_b, H);
        Y->g2 = dupf(w[l].ln2_g, H); Y->be2 = dupf(w[l].ln2_b, H);
        Y->zero_h = (float *)calloc(F > 3 * H ? F : 3 * H, sizeof(float));
        if (Y->mode & ORC_MHA_INT8) {
            float *sw = (float *)malloc(sizeof(float) * 3 * H);
            Y->qkv_t = quant_transposed(w[l].w_qkv, 3 * H, H, sw);
            Y->m_qkv = (float *)malloc(sizeof(float) * 3 * H);
            Y->b_qkv_q = (float *)malloc(sizeof(float) * 3 * H);
            float so[3] = { Y->s.q, Y->s.k, Y->s.v };
            for (int part = 0; part < 3; part++)   /* Q, K and V thirds have their own output steps */
                orc_fold_requant(Y->s.x, sw + part * H, Y->b_qkv + part * H, so[part], H,
                                 Y->m_qkv + part * H, Y->b_qkv_q + part * H);
            Y->o_t = quant_transposed(w[l].w_o, H, H, sw);
            Y->m_o = (float *)malloc(sizeof(float) * H);
            float *tmp = (float *)malloc(sizeof(float) * H);
            orc_fold_requant(Y->s.ctx, sw, NULL, Y->s.attn_out, H, Y->m_o, tmp);
            free(tmp); free(sw);
        } else {
            Y->qkv_f = transpose_f16_to_f32(w[l].w_qkv, 3 * H, H);
            Y->o_f = transpose_f16_to_f32(w[l].w_o, H, H);
        }
        if (Y->mode & ORC_FFN_INT8) {
            float *sw = (float *)malloc(sizeof(float) * (F > H ? F : H));
            Y->f1_t = quant_transposed(w[l].w_ffn1, F, H, sw);
            Y->m_f1 = (float *)malloc(sizeof(float) * F);
            orc_fold_dequant(Y->s.ffn_in, sw, F, Y->m_f1);
            Y->f2_t = quant_transposed(w[l].w_ffn2, H, F, sw);
            Y->m_f2 = (float *)malloc(sizeof(float) * H);
            float *tmp = (float *)malloc(sizeof(float) * H);
            orc_fold_requant(Y->s.ffn_mid, sw, NULL, Y->s.ffn_out, H, Y->m_f2, tmp);
            free(tmp); free(sw);
        } else {
            Y->f1_f = transpose_f16_to_f32(w[l].w_ffn1, F, H);
            Y->f2_f = transpose_f16_to_f32(w[l].w_ffn2, H, F);
        }
    }
    return E;
}

ORC_API void orc_encoder_destroy(orc_encoder *E)
{
    if (!E) return;
    for (int l = 0; l < E->cfg.layers; l++) {
        orc_layer *Y = &E->L[l];
        free(Y->qkv_t); free(Y->o_t); free(Y->f1_t); free(Y->f2_t);
        free(Y->m_qkv); free(Y->b_qkv_q); free(Y->m_o); free(Y->m_f1); free(Y->m_f2); free(Y->zero_h);
        free(Y->qkv_f); free(Y->o_f); free(Y->f1_f); free(Y->f2_f);
        free(Y->b_qkv); free(Y->b_o); free(Y->b_f1); free(Y->b_f2);
        free(Y->g1); free(Y->be1); free(Y->g2); free(Y->be2);
    }
    free(E->L); free(E);
}

/* Optional copies of one layer's tensors for the first processed sequence of a
 * call (pass B = 1 to choose it).  Any pointer may be NULL.  Each buffer holds
 * n rows of int8 or fp16, whichever the layer's mode produces at that point.  */
typedef struct {
    int32_t layer;
    void *x, *qkv, *ctx, *attn_out, *h1, *ffn_mid, *ffn_out, *y;
} orc_taps;

static void tap(void *dst, const void *src, size_t bytes) { if (dst) memcpy(dst, src, bytes); }

/* One sequence of n tokens through all layers.  The step order inside a layer
 * follows Section 3.2: QKV GEMM, attention, attention-output GEMM, fused
 * bias+residual+LayerNorm(+quant), FFN1 GEMM + bias + GELU (+quant), FFN2 GEMM,
 * fused bias+residual+LayerNorm(+quant unless the consumer is floating point). */
typedef struct { const orc_embedding *emb; const int32_t *token_ids, *segment_ids; } orc_ids;

static void forward_sequence(const orc_encoder *E, const uint16_t *hidden, const orc_ids *ids, int n, uint16_t *out,
                             const orc_taps *taps)
{
    const int H = E->cfg.hidden, F = E->cfg.ffn, heads = E->cfg.heads, Lc = E->cfg.layers;
    const float eps = E->cfg.ln_eps;
    size_t nH = (size_t)n * H;
    void *x = malloc(nH * 2), *qkv = malloc(nH * 3 * 2), *ctx = malloc(nH * 2), *ao = malloc(nH * 2);
    void *h1 = malloc(nH * 2), *f1 = malloc((size_t)n * F * 2), *f2 = malloc(nH * 2), *y = malloc(nH * 2);
    int32_t *acc = (int32_t *)malloc(sizeof(int32_t) * (size_t)n * (F > 3 * H ? F : 3 * H));
    int32_t cu[2] = { 0, n };

    /* entry: the producer of a tensor quantises it with its consumer's step */
    if (ids)                           /* the Embedding kernel is that producer */
        orc_embed_ln(ids->emb, ids->token_ids, ids->segment_ids, n, H, x, (E->L[0].mode & ORC_MHA_INT8) != 0, E->L[0].s.x);
    else if (E->L[0].mode & ORC_MHA_INT8) orc_quantize_f16(hidden, nH, E->L[0].s.x, (int8_t *)x);
    else memcpy(x, hidden, nH * 2);

    for (int l = 0; l < Lc; l++) {
        const orc_layer *Y = &E->L[l];
        const orc_layer_scales *s = &Y->s;
        int mha8 = (Y->mode & ORC_MHA_INT8) != 0, ffn8 = (Y->mode & ORC_FFN_INT8) != 0;
        int pu = (Y->mode & ORC_P_UNSIGNED) != 0;
        int last = (l == Lc - 1);
        int next8 = !last && (E->L[l + 1].mode & ORC_MHA_INT8);
        int tp = taps && taps->layer == l;
        if (tp) tap(taps->x, x, nH * (mha8 ? 1 : 2));

        if (mha8) {
            gemm_i8_t((const int8_t *)x, Y->qkv_t, acc, n, 3 * H, H);
            orc_epilogue_requant(acc, n, 3 * H, Y->m_qkv, Y->b_qkv_q, (int8_t *)qkv);
            if (Y->mode & ORC_P_FP16)
                orc_attention_i8_p16((const int8_t *)qkv, cu, 1, H, heads, s->q, s->k, s->v, s->ctx, (int8_t *)ctx);
            else
                orc_attention_i8((const int8_t *)qkv, cu, 1, H, heads, s->q, s->k, s->v, s->p, s->ctx, pu, (int8_t *)ctx, NULL);
            gemm_i8_t((const int8_t *)ctx, Y->o_t, acc, n, H, H);
            orc_epilogue_requant(acc, n, H, Y->m_o, Y->zero_h, (int8_t *)ao);
        } else {
            gemm_f16_t((const uint16_t *)x, Y->qkv_f, Y->b_qkv, 0, (uint16_t *)qkv, n, 3 * H, H);
            orc_attention_f16((const uint16_t *)qkv, cu, 1, H, heads, (uint16_t *)ctx);
            gemm_f16_t((const uint16_t *)ctx, Y->o_f, NULL, 0, (uint16_t *)ao, n, H, H);
        }
        if (tp) { tap(taps->qkv, qkv, nH * 3 * (mha8 ? 1 : 2)); tap(taps->ctx, ctx, nH * (mha8 ? 1 : 2));
                  tap(taps->attn_out, ao, nH * (mha8 ? 1 : 2)); }
        /* the residual is the very tensor the block's first GEMM consumed */
        orc_add_ln(ao, mha8, s->attn_out, Y->b_o, x, mha8, s->x, Y->g1, Y->be1, eps,
                   h1, ffn8, s->ffn_in, n, H);
        if (tp) tap(taps->h1, h1, nH * (ffn8 ? 1 : 2));

        if (ffn8) {
            gemm_i8_t((const int8_t *)h1, Y->f1_t, acc, n, F, H);
            orc_epilogue_gelu_quant(acc, n, F, Y->m_f1, Y->b_f1, s->ffn_mid, (int8_t *)f1);
            gemm_i8_t((const int8_t *)f1, Y->f2_t, acc, n, H, F);
            orc_epilogue_requant(acc, n, H, Y->m_f2, Y->zero_h, (int8_t *)f2);
        } else {
            gemm_f16_t((const uint16_t *)h1, Y->f1_f, Y->b_f1, 1, (uint16_t *)f1, n, F, H);
            gemm_f16_t((const uint16_t *)f1, Y->f2_f, NULL, 0, (uint16_t *)f2, n, H, F);
        }
        if (tp) { tap(taps->ffn_mid, f1, (size_t)n * F * (ffn8 ? 1 : 2)); tap(taps->ffn_out, f2, nH * (ffn8 ? 1 : 2)); }
        orc_add_ln(f2, ffn8, s->ffn_out, Y->b_f2, h1, ffn8, s->ffn_in, Y->g2, Y->be2, eps,
                   y, next8, next8 ? E->L[l + 1].s.x : 1.0f, n, H);
        if (tp) tap(taps->y, y, nH * (next8 ? 1 : 2));
        void *tmp = x; x = y; y = tmp;
    }
    memcpy(out, x, nH * 2);      /* the last layer always leaves fp16 */
    free(x); free(qkv); free(ctx); free(ao); free(h1); free(f1); free(f2); free(y); free(acc);
}

/* hidden, out: fp16 [B,S,H]; lens[b] valid tokens at the start of row block b
 * (right padding).  Padded output rows are zero.  Sequences are independent
 * because every scale is fixed (Appendix B), so they run on separate threads. */
ORC_API int orc_encoder_forward(const orc_encoder *E, const uint16_t *hidden, const int32_t *lens,
                                int B, int S, uint16_t *out, int nthreads, const orc_taps *taps)
{
    const int H = E->cfg.hidden;
    for (int b = 0; b < B; b++) if (lens[b] < 1 || lens[b] > S) return -1;
    memset(out, 0, (size_t)B * S * H * 2);
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    #pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; b++)
        forward_sequence(E, hidden + (size_t)b * S * H, NULL, lens[b], out + (size_t)b * S * H,
                         (taps && b == 0) ? taps : NULL);
    return 0;
}

/* The same with the Embedding kernel in front: token_ids, segment_ids int32 [B,S] (segment_ids may be
 * NULL); the first lens[b] ids of row b are used.                                                  */
ORC_API int orc_encoder_forward_ids(const orc_encoder *E, const orc_embedding *emb, const int32_t *token_ids,
                                    const int32_t *segment_ids, const int32_t *lens, int B, int S, uint16_t *out,
                                    int nthreads)
{
    const int H = E->cfg.hidden;
    for (int b = 0; b < B; b++) if (lens[b] < 1 || lens[b] > S) return -1;
    memset(out, 0, (size_t)B * S * H * 2);
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    #pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; b++) {
        orc_ids ids = { emb, token_ids + (size_t)b * S, segment_ids ? segment_ids + (size_t)b * S : NULL };
        forward_sequence(E, NULL, &ids, lens[b], out + (size_t)b * S * H, NULL);
    }
    return 0;
}

ORC_API int orc_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------------ */
/* Unquantised reference forward in binary64 and the min-max calibration      */
/* (Table 2 caption / Section 4.1: a min-max calibrator yields the scales;    */
/* Appendix B: they are computed once and then fixed).  Reading: the float    */
/* model is run without any rounding on the calibration batch and each        */
/* tensor's absolute maximum over all its tokens is recorded.                 */
/* ------------------------------------------------------------------------ */
static void gemm_ref(const double *A, const uint16_t *W, const float *bias, double *C, int M, int N, int K)
{
    float *Wt = transpose_f16_to_f32(W, N, K);
    for (int t = 0; t < M; t++) {
        double *c = C + (size_t)t * N;
        for (int n = 0; n < N; n++) c[n] = 0.0;
        for (int k = 0; k < K; k++) {
            double a = A[(size_t)t * K + k];
            const float *w = Wt + (size_t)k * N;
            for (int n = 0; n < N; n++) c[n] += a * (double)w[n];
        }
        if (bias) for (int n = 0; n < N; n++) c[n] += (double)bias[n];
    }
    free(Wt);
}

static void ln_ref(const double *z, const float *g, const float *b, double eps, double *y, int M, int H)
{
    for (int t = 0; t < M; t++) {
        const double *r = z + (size_t)t * H;
        double mu = 0.0, var = 0.0;
        for (int c = 0; c < H; c++) mu += r[c];
        mu /= H;
        for (int c = 0; c < H; c++) var += (r[c] - mu) * (r[c] - mu);
        var /= H;
        double rstd = 1.0 / sqrt(var + eps);
        for (int c = 0; c < H; c++) y[(size_t)t * H + c] = (r[c] - mu) * rstd * (double)g[c] + (double)b[c];
    }
}

static void upd(float *slot, const double *v, size_t n)
{
    double m = *slot;
    for (size_t i = 0; i < n; i++) { double a = fabs(v[i]); if (a > m) m = a; }
    *slot = (float)m;
}

/* absmax: [layers][10] in the order of orc_layer_scales, updated in place (start from 0). */
static void reference_sequence(const orc_config *cfg, const orc_layer_weights *w, const uint16_t *hidden, int n,
                               double *out, float *absmax)
{
    int H = cfg->hidden, F = cfg->ffn, heads = cfg->heads, d = H / heads;
    size_t nH = (size_t)n * H;
    double *x = (double *)malloc(sizeof(double) * nH), *qkv = (double *)malloc(sizeof(double) * nH * 3);
    double *ctx = (double *)malloc(sizeof(double) * nH), *ao = (double *)malloc(sizeof(double) * nH);
    double *z = (double *)malloc(sizeof(double) * nH), *h1 = (double *)malloc(sizeof(double) * nH);
    double *f1 = (double *)malloc(sizeof(double) * (size_t)n * F), *f2 = (double *)malloc(sizeof(double) * nH);
    double *p = (double *)malloc(sizeof(double) * n);
    for (size_t i = 0; i < nH; i++) x[i] = (double)h2f(hidden[i]);
    for (int l = 0; l < cfg->layers; l++) {
        float local[10] = { 0 };
        float *am = absmax ? local : NULL;
        if (am) upd(&am[0], x, nH);
        gemm_ref(x, w[l].w_qkv, w[l].b_qkv, qkv, n, 3 * H, H);
        if (am) for (int t = 0; t < n; t++) for (int part = 0; part < 3; part++)
            upd(&am[1 + part], qkv + (size_t)t * 3 * H + part * H, H);
        for (int h = 0; h < heads; h++)
            for (int i = 0; i < n; i++) {
                double mx = -INFINITY, S = 0.0;
                for (int j = 0; j < n; j++) {
                    double a = 0.0;
                    for (int c = 0; c < d; c++)
                        a += qkv[(size_t)i * 3 * H + h * d + c] * qkv[(size_t)j * 3 * H + H + h * d + c];
                    p[j] = a / sqrt((double)d);
                    if (p[j] > mx) mx = p[j];
                }
                for (int j = 0; j < n; j++) { p[j] = exp(p[j] - mx); S += p[j]; }
                for (int j = 0; j < n; j++) p[j] /= S;
                if (am) upd(&am[4], p, n);
                for (int c = 0; c < d; c++) {
                    double O = 0.0;
                    for (int j = 0; j < n; j++) O += p[j] * qkv[(size_t)j * 3 * H + 2 * H + h * d + c];
                    ctx[(size_t)i * H + h * d + c] = O;
                }
            }
        if (am) upd(&am[5], ctx, nH);
        gemm_ref(ctx, w[l].w_o, NULL, ao, n, H, H);
        if (am) upd(&am[6], ao, nH);
        for (size_t i = 0; i < nH; i++) z[i] = ao[i] + (double)w[l].b_o[i % H] + x[i];
        ln_ref(z, w[l].ln1_g, w[l].ln1_b, (double)cfg->ln_eps, h1, n, H);
        if (am) upd(&am[7], h1, nH);
        gemm_ref(h1, w[l].w_ffn1, w[l].b_ffn1, f1, n, F, H);
        for (size_t i = 0; i < (size_t)n * F; i++) f1[i] = 0.5 * f1[i] * (1.0 + erf(f1[i] * 0.70710678118654752440));
        if (am) upd(&am[8], f1, (size_t)n * F);
        gemm_ref(f1, w[l].w_ffn2, NULL, f2, n, H, F);
        if (am) upd(&am[9], f2, nH);
        for (size_t i = 0; i < nH; i++) z[i] = f2[i] + (double)w[l].b_ffn2[i % H] + h1[i];
        ln_ref(z, w[l].ln2_g, w[l].ln2_b, (double)cfg->ln_eps, x, n, H);
        if (am) {
            #pragma omp critical
            for (int i = 0; i < 10; i++) if (local[i] > absmax[l * 10 + i]) absmax[l * 10 + i] = local[i];
        }
    }
    if (out) memcpy(out, x, sizeof(double) * nH);
    free(x); free(qkv); free(ctx); free(ao); free(z); free(h1); free(f1); free(f2); free(p);
}

/* out: binary64 [B,S,H] (may be NULL); absmax: float [layers*10] (may be NULL; caller zeroes it). */
ORC_API int orc_reference_forward(const orc_config *cfg, const orc_layer_weights *w, const uint16_t *hidden,
                                  const int32_t *lens, int B, int S, double *out, float *absmax, int nthreads)
{
    int H = cfg->hidden;
    for (int b = 0; b < B; b++) if (lens[b] < 1 || lens[b] > S) return -1;
    if (out) memset(out, 0, sizeof(double) * (size_t)B * S * H);
#ifdef _OPENMP
    if (nthreads > 0) omp_set_num_threads(nthreads);
#endif
    #pragma omp parallel for schedule(dynamic, 1)
    for (int b = 0; b < B; b++)
        reference_sequence(cfg, w, hidden + (size_t)b * S * H, lens[b], out ? out + (size_t)b * S * H : NULL, absmax);
    return 0;
}

/* scale = absmax / 127 in binary32 */
ORC_API void orc_scales_from_absmax(const float *absmax, int n, float *scales)
{
    for (int i = 0; i < n; i++) scales[i] = absmax[i] / 127.0f;
}
