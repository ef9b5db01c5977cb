// Memory-bound kernels of the encoder: the fused dequantise + bias + residual + LayerNorm (+ quantise)
// step of Section 3.2, padding removal on entry, entry quantisation, per-channel weight quantisation
// and epilogue-table folding at create time, and the absmax taps of the min-max calibration.
// All of them move each byte once with coalesced 4..16-byte accesses; reductions stay inside a wave.
#include "samp_common.h"
#include <hip/hip_ext.h>
#include <algorithm>

namespace samp {
namespace {

// ---------------------------------------------------------------------------------------------
// Fused step: 16 lanes per token row (4 rows per wave); a lane owns 16 consecutive channels of
// every 256-channel slab, so that a row is read with 16-byte (int8) / 32-byte (fp16) accesses
// and its statistics are reduced inside one DPP row (four register-to-register steps).
//   z = fmaf(in_q, s_in, bias) or in + bias;  z = fmaf(res_q, s_res, z) or z + res
//   mean / variance in binary64 (two passes over registers), rounded once to binary32
//   y = fmaf((z - mu) * rstd, gamma, beta);  out = rne(y / s_out) or fp16(y)
// ---------------------------------------------------------------------------------------------
constexpr int LN_ROWS = 8;               // token rows per block of the LayerNorm step (16 lanes each): small blocks slot in beside the other group's kernels

template <int CTRL> __device__ __forceinline__ int dpp_mov(int v)
{ return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xf, 0xf, true); }

template <int CTRL> __device__ __forceinline__ double dpp_mov(double v)
{
    const long long b = __double_as_longlong(v);
    const int lo = dpp_mov<CTRL>((int)b), hi = dpp_mov<CTRL>((int)(b >> 32));
    return __longlong_as_double(((long long)hi << 32) | (unsigned)lo);
}

// sum over the 16 lanes of a DPP row; every lane ends with the same bits (the adds commute)
__device__ __forceinline__ double row16_sum(double v)
{
    v += dpp_mov<0xB1>(v);            // quad_perm [1,0,3,2]
    v += dpp_mov<0x4E>(v);            // quad_perm [2,3,0,1]
    v += dpp_mov<0x141>(v);           // row_half_mirror
    v += dpp_mov<0x140>(v);           // row_mirror
    return v;
}
__device__ __forceinline__ float row16_max(float v)
{
    v = __builtin_fmaxf(v, __int_as_float(dpp_mov<0xB1>(__float_as_int(v))));
    v = __builtin_fmaxf(v, __int_as_float(dpp_mov<0x4E>(__float_as_int(v))));
    v = __builtin_fmaxf(v, __int_as_float(dpp_mov<0x141>(__float_as_int(v))));
    v = __builtin_fmaxf(v, __int_as_float(dpp_mov<0x140>(__float_as_int(v))));
    return v;
}

template <bool I8> __device__ __forceinline__ void load16(const void *p, size_t elem, float (&v)[16])
{
    if (I8) {
        const v4i q = *reinterpret_cast<const v4i *>((const int8_t *)p + elem);
#pragma unroll
        for (int e = 0; e < 16; e++) v[e] = (float)(int8_t)(q[e >> 2] >> (8 * (e & 3)));
    } else {
        const v8h a = *reinterpret_cast<const v8h *>((const __half *)p + elem);
        const v8h b = *reinterpret_cast<const v8h *>((const __half *)p + elem + 8);
#pragma unroll
        for (int e = 0; e < 8; e++) { v[e] = (float)a[e]; v[8 + e] = (float)b[e]; }
    }
}

// Second half of a LayerNorm row held by 16 lanes (z: this lane's channels, sum: its partial sum):
// binary64 mean and variance, binary32 normalisation, output as int8 codes or fp16 at element
// offset obase, optional running absmax of the fp16 output.
// WHOLE: H == 256 NJ, every lane owns NJ full sections and the tests against H fold away (with them the branches
// that keep the compiler from requesting all sections of a row at once).
template <int NJ, bool OUT_I8, bool WHOLE = false>
__device__ __forceinline__ void ln_finish(const float (&z)[NJ][16], double sum, int H, int sub, const float *gamma,
                                          const float *beta, float eps, float s_out, void *out, size_t obase, float *absmax_out)
{
    const double mu = row16_sum(sum) / (double)H;
    double sq = 0.0;
#pragma unroll
    for (int j = 0; j < NJ; j++) {
        if (WHOLE || j * 256 + sub * 16 < H) {
#pragma unroll
            for (int e = 0; e < 16; e++) { const double d = (double)z[j][e] - mu; sq = __builtin_fma(d, d, sq); }
        }
    }
    const double var = row16_sum(sq) / (double)H;
    const float mu32 = (float)mu;
    const float rstd32 = (float)(1.0 / sqrt(var + (double)eps));
    const float inv_s = OUT_I8 ? 1.0f / s_out : 0.0f;
    float amax = 0.0f;
#pragma unroll
    for (int j = 0; j < NJ; j++) {
        const int c = j * 256 + sub * 16;
        if (WHOLE || c < H) {
            float y[16];
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const v4f gg = *reinterpret_cast<const v4f *>(gamma + c + 4 * q);
                const v4f be = *reinterpret_cast<const v4f *>(beta + c + 4 * q);
#pragma unroll
                for (int t = 0; t < 4; t++)
                    y[4 * q + t] = __builtin_fmaf((z[j][4 * q + t] - mu32) * rstd32, gg[t], be[t]);
            }
            if (OUT_I8) {
                v4i o;
#pragma unroll
                for (int q = 0; q < 4; q++)
                    o[q] = pack_codes(code_bits(y[4 * q] * inv_s), code_bits(y[4 * q + 1] * inv_s), code_bits(y[4 * q + 2] * inv_s),
                                      code_bits(y[4 * q + 3] * inv_s));
                *reinterpret_cast<v4i *>((int8_t *)out + obase + c) = o;
            } else {
                v8h h0, h1;
#pragma unroll
                for (int e = 0; e < 8; e++) { h0[e] = to_half(y[e]); h1[e] = to_half(y[8 + e]); }
                *reinterpret_cast<v8h *>((__half *)out + obase + c) = h0;
                *reinterpret_cast<v8h *>((__half *)out + obase + c + 8) = h1;
                if (absmax_out) {
#pragma unroll
                    for (int e = 0; e < 8; e++)
                        amax = __builtin_fmaxf(amax, __builtin_fmaxf(__builtin_fabsf((float)h0[e]), __builtin_fabsf((float)h1[e])));
                }
            }
        }
    }
    if (!OUT_I8 && absmax_out) {
        amax = row16_max(amax);
        if (sub == 0) atomicMax(reinterpret_cast<int *>(absmax_out), __float_as_int(amax));   // values >= 0
    }
}

template <int NJ, bool IN_I8, bool RES_I8, bool OUT_I8, bool WHOLE>
__global__ __launch_bounds__(16 * LN_ROWS) void add_ln_kernel(AddLnArgs a)
{
    const int M = a.rows.dev_rows ? *a.rows.dev_rows : a.rows.host_rows;
    const int nblk = (M + LN_ROWS - 1) / LN_ROWS;
    if ((int)blockIdx.x >= nblk) return;
    const int row = xcd_contiguous(blockIdx.x, nblk) * LN_ROWS + (threadIdx.x >> 4);   // XCD x: x-th eighth of the rows
    if (row >= M) return;                               // whole 16-lane rows leave together
    const int sub = threadIdx.x & 15, H = a.H;
    const size_t base = (size_t)row * H;
    const int out_row = a.row_map ? a.row_map[row] : row;        // requested with the row's data, not after it

    float z[NJ][16];
    double sum = 0.0;
#pragma unroll
    for (int j = 0; j < NJ; j++) {
        const int c = j * 256 + sub * 16;
        if (WHOLE || c < H) {
            float x[16], r[16];
            load16<IN_I8>(a.in, base + c, x);
            load16<RES_I8>(a.res, base + c, r);
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const v4f bb = *reinterpret_cast<const v4f *>(a.bias + c + 4 * q);
#pragma unroll
                for (int t = 0; t < 4; t++) {
                    const int e = 4 * q + t;
                    const float u = IN_I8 ? __builtin_fmaf(x[e], a.s_in, bb[t]) : x[e] + bb[t];
                    z[j][e] = RES_I8 ? __builtin_fmaf(r[e], a.s_res, u) : u + r[e];
                    sum += (double)z[j][e];
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < 16; e++) z[j][e] = 0.0f;
        }
    }
    ln_finish<NJ, OUT_I8, WHOLE>(z, sum, H, sub, a.gamma, a.beta, a.eps, a.s_out, a.out,
                                 (size_t)out_row * H, a.absmax_out);
}

template <int NJ>
hipError_t launch_add_ln_nj(const AddLnArgs &a, hipStream_t st, const Timing *tm)
{
    dim3 grid((a.rows.host_rows + LN_ROWS - 1) / LN_ROWS), block(16 * LN_ROWS);
    // width 768 has an instance without tests against H (at 1024 the requests of a whole row in flight take so many
    // registers that the forward gets slower)
    constexpr bool WHOLE_WIDTHS = NJ == 3;
#define SAMP_LN_CASE(I, R, O)                                                                              \
    if (a.in_i8 == I && a.res_i8 == R && a.out_i8 == O) {                                                  \
        if (WHOLE_WIDTHS && a.H == 256 * NJ) launch_kernel(add_ln_kernel<NJ, I, R, O, WHOLE_WIDTHS>, grid, block, 0, st, tm, a); \
        else launch_kernel(add_ln_kernel<NJ, I, R, O, false>, grid, block, 0, st, tm, a);                  \
        return hipGetLastError();                                                                          \
    }
    SAMP_LN_CASE(true, true, true) SAMP_LN_CASE(true, true, false) SAMP_LN_CASE(false, false, true)
    SAMP_LN_CASE(false, false, false) SAMP_LN_CASE(true, false, true) SAMP_LN_CASE(true, false, false)
    SAMP_LN_CASE(false, true, true) SAMP_LN_CASE(false, true, false)
#undef SAMP_LN_CASE
    return hipErrorInvalidValue;
}

// ---------------------------------------------------------------------------------------------
// Embedding kernel (Section 3.1: the token, segment and position embeddings are summed in one kernel;
// Section 3.2: a quantised first block receives INT8 from it directly).  BERT's embedding ends with
// a LayerNorm, done here too.  16 lanes per (b, s) position; valid positions write packed row
// cu[b] + s (and remember where they came from), padded ones zero their row of the final output.
//   z = (tok[id] + seg[sid]) + pos[s]  in binary32;  out = LayerNorm(z) as fp16 or rne(y / s_out).
// Ids outside their table are clamped into it, so no id can make the kernel read out of bounds.
// ---------------------------------------------------------------------------------------------
template <int NJ, bool OUT_I8>
__global__ __launch_bounds__(256) void embed_ln_kernel(EmbedArgs a)
{
    const int rowid = blockIdx.x * 16 + (threadIdx.x >> 4);
    if (rowid >= a.B * a.S) return;
    const int sub = threadIdx.x & 15, H = a.H;
    const int b = rowid / a.S, s = rowid - b * a.S;
    int t = rowid;
    if (a.cu) {
        const int t0 = a.cu[b], n = a.cu[b + 1] - t0;
        if (s >= n) {
            if (a.out_zero_pad)
                for (int c = sub * 8; c < H; c += 128) *reinterpret_cast<v4i *>(a.out_zero_pad + (size_t)rowid * H + c) = v4i{0, 0, 0, 0};
            return;
        }
        t = t0 + s;
        if (sub == 0 && a.row_map) a.row_map[t] = rowid;
    }
    const int id = min(max(a.token_ids[rowid], 0), a.vocab - 1);
    const int sid = a.segment_ids ? min(max(a.segment_ids[rowid], 0), a.segments - 1) : 0;
    const int pid = min(s, a.positions - 1);
    float z[NJ][16];
    double sum = 0.0;
#pragma unroll
    for (int j = 0; j < NJ; j++) {
        const int c = j * 256 + sub * 16;
        if (c < H) {
            float x[16], g[16], p[16];
            load16<false>(a.tok, (size_t)id * H + c, x);
            load16<false>(a.seg, (size_t)sid * H + c, g);
            load16<false>(a.pos, (size_t)pid * H + c, p);
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const float u = x[e] + g[e];
                z[j][e] = u + p[e];
                sum += (double)z[j][e];
            }
        } else {
#pragma unroll
            for (int e = 0; e < 16; e++) z[j][e] = 0.0f;
        }
    }
    ln_finish<NJ, OUT_I8>(z, sum, H, sub, a.gamma, a.beta, a.eps, a.s_out, a.out, (size_t)t * H, nullptr);
}

template <int NJ>
hipError_t launch_embed_ln_nj(const EmbedArgs &a, hipStream_t st, const Timing *tm)
{
    dim3 grid((a.B * a.S + 15) / 16), block(256);
    if (a.out_i8) launch_kernel(embed_ln_kernel<NJ, true>, grid, block, 0, st, tm, a);
    else launch_kernel(embed_ln_kernel<NJ, false>, grid, block, 0, st, tm, a);
    return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Sequence offsets: cu[b] = number of valid tokens before sequence b (exclusive prefix sum of the
// mask's row sums), cu[B] = T.  One block; wave w sums the rows w, w+16, ...
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(1024) void seq_offsets_kernel(const int *__restrict__ mask, int B, int S, int *__restrict__ cu)
{
    extern __shared__ int len[];                    // [B]
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int b = wave; b < B; b += 16) {
        int s = 0;
        if (mask) { for (int i = lane; i < S; i += 64) s += mask[(size_t)b * S + i] != 0; }
        else s = (lane == 0) ? S : 0;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
        if (lane == 0) len[b] = s;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int run = 0;
        for (int b = 0; b < B; b++) { cu[b] = run; run += len[b]; }
        cu[B] = run;
    }
}

// Padding removal: one wave per (b, s) row.  Valid rows are copied (or quantised) to packed row
// cu[b] + s and remember where they came from; padded rows zero the matching row of the final output.
__global__ __launch_bounds__(256) void pack_rows_kernel(const __half *__restrict__ hidden, const int *__restrict__ cu,
                                                        int B, int S, int H, float s_x, void *__restrict__ packed,
                                                        int *__restrict__ row_map, __half *__restrict__ out_zero_pad)
{
    const int rowid = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (rowid >= B * S) return;
    const int lane = threadIdx.x & 63;
    const int b = rowid / S, s = rowid - b * S;
    const int t0 = cu[b], n = cu[b + 1] - t0;
    if (s >= n) {
        if (out_zero_pad)
            for (int c = lane * 8; c < H; c += 512) *reinterpret_cast<v4i *>(out_zero_pad + (size_t)rowid * H + c) = v4i{0, 0, 0, 0};
        return;
    }
    const int t = t0 + s;
    if (lane == 0) row_map[t] = rowid;
    const __half *src = hidden + (size_t)rowid * H;
    if (s_x > 0.0f) {
        const float inv_s = 1.0f / s_x;
        for (int c = lane * 8; c < H; c += 512) {
            const v8h v = *reinterpret_cast<const v8h *>(src + c);
            v2i o;
            o.x = pack4(qcode((float)v[0] * inv_s), qcode((float)v[1] * inv_s), qcode((float)v[2] * inv_s), qcode((float)v[3] * inv_s));
            o.y = pack4(qcode((float)v[4] * inv_s), qcode((float)v[5] * inv_s), qcode((float)v[6] * inv_s), qcode((float)v[7] * inv_s));
            *reinterpret_cast<v2i *>((int8_t *)packed + (size_t)t * H + c) = o;
        }
    } else {
        for (int c = lane * 8; c < H; c += 512)
            *reinterpret_cast<v4i *>((__half *)packed + (size_t)t * H + c) = *reinterpret_cast<const v4i *>(src + c);
    }
}

// Entry quantisation without padding removal: code = rne(x * (1/s_x)), 8 elements per thread.
__global__ __launch_bounds__(256) void quantize_rows_kernel(const __half *__restrict__ x, size_t n8, float s_x,
                                                            int8_t *__restrict__ out)
{
    const float inv_s = 1.0f / s_x;
    // one contiguous chunk per block, chunks numbered so that XCD x quantises the x-th eighth of the tensor
    const size_t chunk = (n8 + gridDim.x - 1) / gridDim.x;
    const size_t first = (size_t)xcd_contiguous(blockIdx.x, gridDim.x) * chunk, last = first + chunk < n8 ? first + chunk : n8;
    for (size_t i = first + threadIdx.x; i < last; i += 256) {
        const v8h v = *reinterpret_cast<const v8h *>(x + i * 8);
        v2i o;
        o.x = pack4(qcode((float)v[0] * inv_s), qcode((float)v[1] * inv_s), qcode((float)v[2] * inv_s), qcode((float)v[3] * inv_s));
        o.y = pack4(qcode((float)v[4] * inv_s), qcode((float)v[5] * inv_s), qcode((float)v[6] * inv_s), qcode((float)v[7] * inv_s));
        *reinterpret_cast<v2i *>(out + i * 8) = o;
    }
}

// Per-output-channel weight quantisation (create time): one block per row of W[N,K].
//   s_w = absmax / 127 (1 for an all-zero row), code = rne(w / s_w) with a true binary32 division.
__global__ __launch_bounds__(256) void quantize_weight_kernel(const __half *__restrict__ W, int K, int8_t *__restrict__ Wq,
                                                              float *__restrict__ s_w)
{
    __shared__ float red[4];
    const int n = blockIdx.x, lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const __half *row = W + (size_t)n * K;
    float amax = 0.0f;
    for (int k = threadIdx.x; k < K; k += 256) amax = __builtin_fmaxf(amax, __builtin_fabsf((float)row[k]));
    amax = wave_max(amax);
    if (lane == 0) red[wave] = amax;
    __syncthreads();
    amax = __builtin_fmaxf(__builtin_fmaxf(red[0], red[1]), __builtin_fmaxf(red[2], red[3]));
    const float s = amax > 0.0f ? __fdiv_rn(amax, 127.0f) : 1.0f;
    if (threadIdx.x == 0) s_w[n] = s;
    for (int k = threadIdx.x; k < K; k += 256) Wq[(size_t)n * K + k] = (int8_t)qcode(__fdiv_rn((float)row[k], s));
}

// Epilogue tables: m[n] = s_in * s_w[n] / s_out, b[n] = bias[n] / s_out, formed in binary64 and
// rounded once (s_out = 1 and bias = nullptr give the plain dequantising multiplier).
__global__ void fold_kernel(float s_in, const float *__restrict__ s_w, const float *__restrict__ bias, float s_out, int N,
                            float *__restrict__ m, float *__restrict__ b)
{
    const int n = blockIdx.x * blockDim.x + threadIdx.x;
    if (n >= N) return;
    m[n] = (float)((double)s_in * (double)s_w[n] / (double)s_out);
    if (b) b[n] = bias ? (float)((double)bias[n] / (double)s_out) : 0.0f;
}

// Calibration tap: running absmax of an fp16 [rows, cols] view with leading dimension ld.
__global__ __launch_bounds__(256) void absmax_f16_kernel(const __half *__restrict__ x, int host_rows,
                                                         const int *__restrict__ dev_rows, int cols, int ld,
                                                         float *__restrict__ slot)
{
    const int rows = dev_rows ? *dev_rows : host_rows;
    float amax = 0.0f;
    const int c8 = cols / 8;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < (size_t)rows * c8; i += (size_t)gridDim.x * 256) {
        const size_t r = i / c8, c = (i - r * c8) * 8;
        const v8h v = *reinterpret_cast<const v8h *>(x + r * ld + c);
#pragma unroll
        for (int e = 0; e < 8; e++) amax = __builtin_fmaxf(amax, __builtin_fabsf((float)v[e]));
    }
    amax = wave_max(amax);
    if ((threadIdx.x & 63) == 0) atomicMax(reinterpret_cast<int *>(slot), __float_as_int(amax));
}

// The FFN1 epilogue's decision step on its own: codes = rne(GELU(y) / s_out); optionally also the
// fast-path GELU values, so that their error bound can be checked from outside.
__global__ __launch_bounds__(256) void gelu_quant_kernel(const float *__restrict__ y, size_t n, float inv_s,
                                                         int8_t *__restrict__ codes, float *__restrict__ fast)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n; i += (size_t)gridDim.x * 256) {
        const float v = y[i];
        codes[i] = (int8_t)gelu_quant_code(v, inv_s);
        if (fast) fast[i] = gelu_fast(v);
    }
}

// counts of each byte value: per-block counters in LDS, merged with one global atomic per bin
__global__ __launch_bounds__(256) void code_histogram_kernel(const int8_t *__restrict__ codes, size_t n,
                                                             unsigned long long *__restrict__ hist)
{
    __shared__ unsigned h[256];
    h[threadIdx.x] = 0;
    __syncthreads();
    const size_t nvec = n / 16;
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < nvec; i += (size_t)gridDim.x * 256) {
        const v4i v = reinterpret_cast<const v4i *>(codes)[i];
#pragma unroll
        for (int k = 0; k < 4; k++)
#pragma unroll
            for (int b = 0; b < 4; b++) atomicAdd(&h[((unsigned)v[k] >> (8 * b)) & 0xffu], 1u);
    }
    if (blockIdx.x == 0)
        for (size_t i = nvec * 16 + threadIdx.x; i < n; i += 256) atomicAdd(&h[(unsigned char)codes[i]], 1u);
    __syncthreads();
    if (h[threadIdx.x]) atomicAdd(&hist[threadIdx.x], (unsigned long long)h[threadIdx.x]);
}

__global__ void fill_f32_kernel(float *p, int n, float v)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

}  // namespace

hipError_t launch_add_ln(const AddLnArgs &a, hipStream_t st, const Timing *tm)
{
    const int nj = (a.H + 255) / 256;
    switch (nj) {
    case 1: return launch_add_ln_nj<1>(a, st, tm);
    case 2: return launch_add_ln_nj<2>(a, st, tm);
    case 3: return launch_add_ln_nj<3>(a, st, tm);
    case 4: return launch_add_ln_nj<4>(a, st, tm);
    case 5: return launch_add_ln_nj<5>(a, st, tm);
    case 6: return launch_add_ln_nj<6>(a, st, tm);
    case 7: return launch_add_ln_nj<7>(a, st, tm);
    case 8: return launch_add_ln_nj<8>(a, st, tm);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_quantize_weight(const __half *W, int N, int K, int8_t *Wq, float *s_w, hipStream_t st)
{
    hipLaunchKernelGGL(quantize_weight_kernel, dim3(N), dim3(256), 0, st, W, K, Wq, s_w);
    return hipGetLastError();
}

hipError_t launch_fold(const float *, float s_in, const float *s_w, const float *bias, float s_out, int N, float *m,
                       float *b, hipStream_t st)
{
    hipLaunchKernelGGL(fold_kernel, dim3((N + 255) / 256), dim3(256), 0, st, s_in, s_w, bias, s_out, N, m, b);
    return hipGetLastError();
}

hipError_t launch_embed_ln(const EmbedArgs &a, hipStream_t st, const Timing *tm)
{
    switch ((a.H + 255) / 256) {
    case 1: return launch_embed_ln_nj<1>(a, st, tm);
    case 2: return launch_embed_ln_nj<2>(a, st, tm);
    case 3: return launch_embed_ln_nj<3>(a, st, tm);
    case 4: return launch_embed_ln_nj<4>(a, st, tm);
    case 5: return launch_embed_ln_nj<5>(a, st, tm);
    case 6: return launch_embed_ln_nj<6>(a, st, tm);
    case 7: return launch_embed_ln_nj<7>(a, st, tm);
    case 8: return launch_embed_ln_nj<8>(a, st, tm);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_seq_offsets(const int *mask, int B, int S, int *cu, hipStream_t st)
{
    hipLaunchKernelGGL(seq_offsets_kernel, dim3(1), dim3(1024), (size_t)B * sizeof(int), st, mask, B, S, cu);
    return hipGetLastError();
}

hipError_t launch_pack_rows(const __half *hidden, const int *cu, int B, int S, int H, float s_x, void *packed,
                            int *row_map, __half *out_zero_pad, hipStream_t st, const Timing *tm)
{
    dim3 grid((B * S + 3) / 4), block(256);
    launch_kernel(pack_rows_kernel, grid, block, 0, st, tm,
                          hidden, cu, B, S, H, s_x, packed, row_map, out_zero_pad);
    return hipGetLastError();
}

hipError_t launch_quantize_rows(const __half *x, size_t n, float s_x, int8_t *out, hipStream_t st, const Timing *tm)
{
    const size_t n8 = n / 8;
    size_t blocks = (n8 + 255) / 256;
    if (blocks > 8192) blocks = 8192;
    launch_kernel(quantize_rows_kernel, dim3((unsigned)blocks), dim3(256), 0, st, tm, x, n8, s_x, out);
    return hipGetLastError();
}

hipError_t launch_absmax_f16(const __half *x, Rows rows, int cols, int ld, float *slot, hipStream_t st)
{
    size_t work = (size_t)rows.host_rows * (cols / 8);
    size_t blocks = (work + 255) / 256;
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(absmax_f16_kernel, dim3((unsigned)blocks), dim3(256), 0, st, x, rows.host_rows, rows.dev_rows, cols,
                       ld, slot);
    return hipGetLastError();
}

hipError_t launch_gelu_quant(const float *y, size_t n, float inv_s, int8_t *codes, float *fast, hipStream_t st)
{
    size_t blocks = (n + 255) / 256;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(gelu_quant_kernel, dim3((unsigned)blocks), dim3(256), 0, st, y, n, inv_s, codes, fast);
    return hipGetLastError();
}

hipError_t launch_code_histogram(const int8_t *codes, size_t n, unsigned long long *hist, hipStream_t st)
{
    const size_t blocks = std::min<size_t>((n / 16 + 255) / 256 + 1, 2048);
    hipLaunchKernelGGL(code_histogram_kernel, dim3((unsigned)blocks), dim3(256), 0, st, codes, n, hist);
    return hipGetLastError();
}

hipError_t launch_fill_f32(float *p, int n, float v, hipStream_t st)
{
    hipLaunchKernelGGL(fill_f32_kernel, dim3((n + 255) / 256), dim3(256), 0, st, p, n, v);
    return hipGetLastError();
}

}  // namespace samp
