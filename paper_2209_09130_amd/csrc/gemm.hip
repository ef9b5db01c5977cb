// INT8 and FP16 "NT" GEMMs on gfx950 matrix cores with fused epilogues (Section 3.2: the four
// GEMMs of a layer run as INT8 with int32 accumulation or as FP16; quantise / dequantise, bias and
// GELU are fused into the producing kernel so that only int8 or fp16 tensors reach memory).
//
//   C[m,n] = sum_k A[m,k] * W[n,k]      A [M,K] and W [N,K] both K-contiguous.
//
// Byte geometry is the same for both element types: one MFMA consumes 32 bytes of K per row
// (v_mfma_i32_32x32x32_i8: 32 int8; v_mfma_f32_32x32x16_f16: 16 fp16), 16 bytes per lane.  The
// weight rows are the MFMA's first operand and the activation rows its second, so that in the
// 32x32 result a lane owns ONE token row and four consecutive output channels per register
// group -- which is what the per-channel epilogue tables and the packed int8/fp16 stores want.
//
// Block tile 128 (tokens) x 128 (channels), 4 waves in 2x2, wave tile 64x64 = 2x2 MFMA tiles.
// K is consumed 64 bytes per step through double-buffered LDS tiles whose 16-byte chunks are
// XOR-swizzled so that both the 16-byte stores and the ds_read_b128 operand fetches are spread
// over all banks.
#include "samp_common.h"

namespace samp {
namespace {

constexpr int BM = 128, BN = 128, BKB = 64;      // BKB: bytes of K per main-loop step
constexpr int NTHREADS = 256;
constexpr int TILE_BYTES = 128 * BKB;            // one operand tile in LDS

// swizzle of the 16-byte chunk index inside a 64-byte LDS row
__device__ __forceinline__ int swz(int row) { return ((row >> 1) & 3) ^ ((row >> 3) & 1); }

struct I8 {
    typedef v16i acc_t;
    static constexpr int ELEM = 1;
    __device__ static __forceinline__ acc_t mma(v4i a, v4i b, acc_t c)
    { return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, c, 0, 0, 0); }
};
struct F16 {
    typedef v16f acc_t;
    static constexpr int ELEM = 2;
    __device__ static __forceinline__ acc_t mma(v4i a, v4i b, acc_t c)
    { return __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), c, 0, 0, 0); }
};

// ---- epilogues: turn 4 accumulators (one token row, channels n..n+3) into stored output ---------
struct EpiRawI32 {                                // test hook: the exact int32 accumulators
    int32_t *out; int N;
    static constexpr int OUT_BYTES = 4;
    static constexpr bool STAGED = false;
    __device__ __forceinline__ void direct(int row, int n, int a0, int a1, int a2, int a3) const
    { *reinterpret_cast<v4i *>(out + (size_t)row * N + n) = v4i{a0, a1, a2, a3}; }
};

struct EpiRequant {                               // code = rne(fmaf(acc, m[n], b[n]))
    const float *m, *b;
    static constexpr int OUT_BYTES = 1;
    static constexpr bool STAGED = true;
    __device__ __forceinline__ int pack(int n, int a0, int a1, int a2, int a3) const
    {
        const v4f mm = *reinterpret_cast<const v4f *>(m + n);
        v4f bb = {0.f, 0.f, 0.f, 0.f};
        if (b) bb = *reinterpret_cast<const v4f *>(b + n);
        return pack4(qcode(__builtin_fmaf((float)a0, mm.x, bb.x)), qcode(__builtin_fmaf((float)a1, mm.y, bb.y)),
                     qcode(__builtin_fmaf((float)a2, mm.z, bb.z)), qcode(__builtin_fmaf((float)a3, mm.w, bb.w)));
    }
};

struct EpiGeluQuant {                             // y = fmaf(acc, m[n], bias[n]); code = rne(GELU(y) / s_out)
    const float *m, *bias; float inv_s;
    static constexpr int OUT_BYTES = 1;
    static constexpr bool STAGED = true;
    __device__ __forceinline__ int pack(int n, int a0, int a1, int a2, int a3) const
    {
        const v4f mm = *reinterpret_cast<const v4f *>(m + n);
        const v4f bb = *reinterpret_cast<const v4f *>(bias + n);
        return pack4(gelu_quant_code(__builtin_fmaf((float)a0, mm.x, bb.x), inv_s),
                     gelu_quant_code(__builtin_fmaf((float)a1, mm.y, bb.y), inv_s),
                     gelu_quant_code(__builtin_fmaf((float)a2, mm.z, bb.z), inv_s),
                     gelu_quant_code(__builtin_fmaf((float)a3, mm.w, bb.w), inv_s));
    }
};

struct EpiF16 {                                   // fp16(act(acc + bias[n]))
    const float *bias; bool gelu;
    static constexpr int OUT_BYTES = 2;
    static constexpr bool STAGED = true;
    __device__ __forceinline__ v2i pack(int n, float a0, float a1, float a2, float a3) const
    {
        if (bias) {
            const v4f bb = *reinterpret_cast<const v4f *>(bias + n);
            a0 += bb.x; a1 += bb.y; a2 += bb.z; a3 += bb.w;
        }
        if (gelu) { a0 = gelu_fast(a0); a1 = gelu_fast(a1); a2 = gelu_fast(a2); a3 = gelu_fast(a3); }
        const v4h h = {to_half(a0), to_half(a1), to_half(a2), to_half(a3)};
        return __builtin_bit_cast(v2i, h);
    }
};

template <class T, class Epi>
__global__ __launch_bounds__(NTHREADS) void gemm_nt_kernel(const char *__restrict__ A, const char *__restrict__ W,
                                                            char *__restrict__ out, Epi epi, int host_rows,
                                                            const int *__restrict__ dev_rows, int N, int Kbytes)
{
    // LDS: [buffer][operand][128 rows][64 bytes]; reused as the output staging tile afterwards
    __shared__ __attribute__((aligned(16))) char lds[2 * 2 * TILE_BYTES + 4096];

    const int M = dev_rows ? *dev_rows : host_rows;
    const int m0 = blockIdx.y * BM, n0 = blockIdx.x * BN;
    if (m0 >= M) return;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 64, wn = (wave & 1) * 64;       // wave tile origin inside the block tile
    const int r = lane & 31, g = lane >> 5;

    // global -> LDS copy assignment: 512 chunks of 16 bytes per operand tile, 2 per thread
    const int crow = tid >> 2, cchunk = tid & 3;
    const char *a_src[2], *w_src[2];
    int lds_off[2];
#pragma unroll
    for (int u = 0; u < 2; u++) {
        const int row = crow + u * 64;
        int am = m0 + row; if (am > M - 1) am = M - 1;            // rows past the end re-read the last row
        a_src[u] = A + (size_t)am * Kbytes + cchunk * 16;
        w_src[u] = W + (size_t)(n0 + row) * Kbytes + cchunk * 16;
        lds_off[u] = row * BKB + ((cchunk ^ swz(row)) << 4);
    }

    typename T::acc_t acc[2][2];                                  // [channel tile][token tile]
#pragma unroll
    for (int i = 0; i < 2; i++)
#pragma unroll
        for (int j = 0; j < 2; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0;

    const int KT = Kbytes / BKB;
    v4i ra[2], rw[2];
#pragma unroll
    for (int u = 0; u < 2; u++) {
        ra[u] = *reinterpret_cast<const v4i *>(a_src[u]);
        rw[u] = *reinterpret_cast<const v4i *>(w_src[u]);
    }
#pragma unroll
    for (int u = 0; u < 2; u++) {
        *reinterpret_cast<v4i *>(lds + lds_off[u]) = ra[u];
        *reinterpret_cast<v4i *>(lds + TILE_BYTES + lds_off[u]) = rw[u];
    }
    __syncthreads();

    for (int kt = 0; kt < KT; kt++) {
        const char *cur = lds + (kt & 1) * 2 * TILE_BYTES;
        if (kt + 1 < KT) {
#pragma unroll
            for (int u = 0; u < 2; u++) {
                ra[u] = *reinterpret_cast<const v4i *>(a_src[u] + (size_t)(kt + 1) * BKB);
                rw[u] = *reinterpret_cast<const v4i *>(w_src[u] + (size_t)(kt + 1) * BKB);
            }
        }
#pragma unroll
        for (int ks = 0; ks < 2; ks++) {
            v4i fa[2], fw[2];
#pragma unroll
            for (int i = 0; i < 2; i++) {
                const int rowa = wm + i * 32 + r, roww = wn + i * 32 + r;
                fa[i] = *reinterpret_cast<const v4i *>(cur + rowa * BKB + (((2 * ks + g) ^ swz(rowa)) << 4));
                fw[i] = *reinterpret_cast<const v4i *>(cur + TILE_BYTES + roww * BKB + (((2 * ks + g) ^ swz(roww)) << 4));
            }
#pragma unroll
            for (int i = 0; i < 2; i++)
#pragma unroll
                for (int j = 0; j < 2; j++) acc[i][j] = T::mma(fw[i], fa[j], acc[i][j]);
        }
        if (kt + 1 < KT) {
            char *nxt = lds + ((kt + 1) & 1) * 2 * TILE_BYTES;
#pragma unroll
            for (int u = 0; u < 2; u++) {
                *reinterpret_cast<v4i *>(nxt + lds_off[u]) = ra[u];
                *reinterpret_cast<v4i *>(nxt + TILE_BYTES + lds_off[u]) = rw[u];
            }
        }
        __syncthreads();
    }

    // Result layout of a 32x32 tile (first operand = channels, second = tokens): lane holds token
    // (lane & 31) and, in register 4q+t, channel 8q + 4(lane >> 5) + t.
    if constexpr (!Epi::STAGED) {
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int j = 0; j < 2; j++) {
                const int row = m0 + wm + j * 32 + r;
                if (row < M) {
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const int n = n0 + wn + i * 32 + 8 * q + 4 * g;
                        epi.direct(row, n, acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                    }
                }
            }
    } else {
        // stage the 128x128 output tile in LDS, then write full rows with 16-byte stores
        constexpr int OB = Epi::OUT_BYTES;
        constexpr int STRIDE = BN * OB + 16;
        static_assert(BM * STRIDE <= 2 * 2 * TILE_BYTES + 4096, "staging tile does not fit");
#pragma unroll
        for (int i = 0; i < 2; i++)
#pragma unroll
            for (int j = 0; j < 2; j++) {
                const int lrow = wm + j * 32 + r;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const int ln = wn + i * 32 + 8 * q + 4 * g;
                    auto v = epi.pack(n0 + ln, acc[i][j][4 * q], acc[i][j][4 * q + 1], acc[i][j][4 * q + 2], acc[i][j][4 * q + 3]);
                    *reinterpret_cast<decltype(v) *>(lds + lrow * STRIDE + ln * OB) = v;
                }
            }
        __syncthreads();
        constexpr int CHUNKS = BN * OB / 16;                      // 16-byte chunks per output row
        constexpr int ROWS_PER_PASS = NTHREADS / CHUNKS;
        const int orow = tid / CHUNKS, ochunk = tid % CHUNKS;
#pragma unroll
        for (int p = 0; p < BM / ROWS_PER_PASS; p++) {
            const int lrow = p * ROWS_PER_PASS + orow;
            if (m0 + lrow < M) {
                const v4i v = *reinterpret_cast<const v4i *>(lds + lrow * STRIDE + ochunk * 16);
                *reinterpret_cast<v4i *>(out + ((size_t)(m0 + lrow) * N + n0) * OB + ochunk * 16) = v;
            }
        }
    }
}

template <class T, class Epi>
hipError_t launch(const void *A, const void *W, void *out, const Epi &epi, Rows rows, int N, int K, hipStream_t st,
                  const Timing *tm)
{
    dim3 grid(N / BN, (rows.host_rows + BM - 1) / BM), block(NTHREADS);
    if (tm)
        hipExtLaunchKernelGGL((gemm_nt_kernel<T, Epi>), grid, block, 0, st, tm->start, tm->stop, 0, (const char *)A,
                              (const char *)W, (char *)out, epi, rows.host_rows, rows.dev_rows, N, K * T::ELEM);
    else
        hipLaunchKernelGGL((gemm_nt_kernel<T, Epi>), grid, block, 0, st, (const char *)A, (const char *)W, (char *)out,
                           epi, rows.host_rows, rows.dev_rows, N, K * T::ELEM);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_gemm_i8(GemmEpilogue epi, const int8_t *A, const int8_t *W, void *out, const float *m, const float *b,
                          float inv_s_out, Rows rows, int N, int K, hipStream_t st, const Timing *tm)
{
    switch (epi) {
    case EPI_RAW_I32: return launch<I8>(A, W, out, EpiRawI32{(int32_t *)out, N}, rows, N, K, st, tm);
    case EPI_REQUANT: return launch<I8>(A, W, out, EpiRequant{m, b}, rows, N, K, st, tm);
    case EPI_GELU_QUANT: return launch<I8>(A, W, out, EpiGeluQuant{m, b, inv_s_out}, rows, N, K, st, tm);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_gemm_f16(const __half *A, const __half *W, const float *bias, bool gelu, __half *out, Rows rows,
                           int N, int K, hipStream_t st, const Timing *tm)
{
    return launch<F16>(A, W, out, EpiF16{bias, gelu}, rows, N, K, st, tm);
}

}  // namespace samp
