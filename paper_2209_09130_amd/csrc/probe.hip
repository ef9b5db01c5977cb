// Measured ceilings of the chip the library runs on, for the benchmark's report: the issue rate of the int8 and
// fp16 matrix instructions the GEMMs are built from (no memory traffic: operands stay in registers), and the rate
// of a plain device copy.  The published peaks (5.0 POP/s int8, 2.5 PFLOP/s fp16, 8 TB/s) assume the full clock;
// under matrix load the clock drops, the more the more operand bits toggle, which is why the probe takes its
// operands either all equal or pseudo-random.
#include "samp_common.h"

namespace samp {
namespace {

template <bool F16>
__global__ __launch_bounds__(256) void mfma_rate_kernel(int iters, unsigned seed, int *sink)
{
    // operands: a per-lane hash (seed != 0) or the same byte pattern everywhere (seed == 0)
    unsigned h = seed ? (threadIdx.x * 2654435761u + blockIdx.x * 40503u + seed) : 0x01010101u;
    v4i a, b;
#pragma unroll
    for (int i = 0; i < 4; i++) {
        if (seed) { h ^= h << 13; h ^= h >> 17; h ^= h << 5; }
        a[i] = F16 ? (int)((h & 0x3fff3fffu) | 0x30003000u) : (int)h;      // fp16: finite values of moderate size
        if (seed) { h ^= h << 13; h ^= h >> 17; h ^= h << 5; }
        b[i] = F16 ? (int)((h & 0x3fff3fffu) | 0x30003000u) : (int)h;
    }
    int out = 0;
    if constexpr (F16) {
        v16f acc[4];
#pragma unroll
        for (int k = 0; k < 4; k++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[k][e] = 0.0f;
        for (int it = 0; it < iters; it++)
#pragma unroll
            for (int k = 0; k < 4; k++)
                acc[k] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, a), __builtin_bit_cast(v8h, b), acc[k], 0, 0, 0);
#pragma unroll
        for (int k = 0; k < 4; k++) out ^= __float_as_int(acc[k][0] + acc[k][7]);
    } else {
        v16i acc[4];
#pragma unroll
        for (int k = 0; k < 4; k++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[k][e] = 0;
        for (int it = 0; it < iters; it++)
#pragma unroll
            for (int k = 0; k < 4; k++) acc[k] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[k], 0, 0, 0);
#pragma unroll
        for (int k = 0; k < 4; k++) out ^= acc[k][0] + acc[k][7];
    }
    if (out == 0x5a5a5a5a) sink[0] = out;                              // keeps the loop alive; practically never taken
}

__global__ __launch_bounds__(256) void copy_kernel(const v4i *__restrict__ src, v4i *__restrict__ dst, size_t n16)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += (size_t)gridDim.x * 256) dst[i] = src[i];
}

// Operand feed without arithmetic: each block walks the K extent of a 128 x 128 GEMM tile in 128-byte stages,
// pulling both operand tiles (32 KiB per stage) from global memory (in practice L2) into a 3-deep LDS ring with
// direct loads, exactly as the GEMM main loops do, and reads one dword of every stage so that nothing is elided.
__global__ __launch_bounds__(256) void feed_rate_kernel(const char *__restrict__ A, const char *__restrict__ W, int kbytes,
                                                        int tiles_n, int *sink)
{
    extern __shared__ __attribute__((aligned(1024))) char ring[];
    constexpr int STAGE = 256 * 128, NS = 3;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int m0 = (blockIdx.x / tiles_n) * 128, n0 = (blockIdx.x % tiles_n) * 128;
    const int steps = kbytes / 128;
    const char *src[8];
#pragma unroll
    for (int j = 0; j < 8; j++) {
        const int row = 8 * (wave + 4 * (j & 3)) + lane / 8;
        const char *base = j < 4 ? A + (size_t)(m0 + row) * kbytes : W + (size_t)(n0 + row) * kbytes;
        src[j] = base + (((lane % 8) ^ (row & 7)) << 4);
    }
    auto issue = [&](int kt) {
        char *st = ring + (kt % NS) * STAGE;
#pragma unroll
        for (int j = 0; j < 8; j++)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[j] + (size_t)kt * 128),
                                             (__attribute__((address_space(3))) void *)(st + (j < 4 ? 0 : 16384) + (wave + 4 * (j & 3)) * 1024),
                                             16, 0, 0);
    };
    int acc = 0;
    for (int s = 0; s < NS - 1; s++)
        if (s < steps) issue(s);
    for (int kt = 0; kt < steps; kt++) {
        if (kt + NS - 2 < steps) asm volatile("s_waitcnt vmcnt(8)" ::: "memory");     // the oldest stage has landed
        else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __syncthreads();
        if (kt + NS - 1 < steps) issue(kt + NS - 1);
        acc += *reinterpret_cast<const int *>(ring + (kt % NS) * STAGE + tid * 16);
    }
    if (acc == 0x12345678) sink[0] = acc;
}

}  // namespace

// bytes per second that `blocks` = (rows / 128) (N / 128) blocks pull into LDS; operands: rows x kbytes and N x kbytes
hipError_t probe_feed_rate(const void *A, const void *W, int rows, int N, int kbytes, int reps, int *sink, hipStream_t st,
                           double *bytes_per_s)
{
    const int tiles_n = N / 128, blocks = tiles_n * (rows / 128);
    const size_t lds = 3 * 256 * 128;
    hipError_t e = hipFuncSetAttribute((const void *)feed_rate_kernel, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipEvent_t e0, e1;
    e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&e1);
    if (e != hipSuccess) { (void)hipEventDestroy(e0); return e; }
    auto launch = [&]() {
        hipLaunchKernelGGL(feed_rate_kernel, dim3(blocks), dim3(256), lds, st, (const char *)A, (const char *)W, kbytes, tiles_n, sink);
    };
    for (int i = 0; i < 3; i++) launch();
    (void)hipEventRecord(e0, st);
    for (int i = 0; i < reps; i++) launch();
    (void)hipEventRecord(e1, st);
    e = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return e;
    *bytes_per_s = (double)blocks * (kbytes / 128) * 32768.0 * reps / (ms * 1e-3);
    return hipGetLastError();
}

// ops (2 per multiply-add) per second over `iters` rounds of four independent MFMAs per wave, 8 waves per SIMD-pair
hipError_t probe_mfma_rate(bool f16, bool random_operands, int iters, int *sink, hipStream_t st, double *ops_per_s)
{
    const int blocks = 2048;
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&e1);
    if (e != hipSuccess) { (void)hipEventDestroy(e0); return e; }
    auto launch = [&](int n) {
        if (f16) hipLaunchKernelGGL(mfma_rate_kernel<true>, dim3(blocks), dim3(256), 0, st, n, random_operands ? 12345u : 0u, sink);
        else hipLaunchKernelGGL(mfma_rate_kernel<false>, dim3(blocks), dim3(256), 0, st, n, random_operands ? 12345u : 0u, sink);
    };
    launch(iters / 8 + 1);                                              // warm-up
    (void)hipEventRecord(e0, st);
    launch(iters);
    (void)hipEventRecord(e1, st);
    e = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return e;
    const double per_mfma = f16 ? 2.0 * 32 * 32 * 16 : 2.0 * 32 * 32 * 32;
    *ops_per_s = (double)blocks * 4 /* waves */ * iters * 4 /* MFMAs */ * per_mfma / (ms * 1e-3);
    return hipGetLastError();
}

hipError_t probe_copy_rate(const void *src, void *dst, size_t bytes, int reps, hipStream_t st, double *bytes_per_s)
{
    hipEvent_t e0, e1;
    hipError_t e = hipEventCreate(&e0);
    if (e != hipSuccess) return e;
    e = hipEventCreate(&e1);
    if (e != hipSuccess) { (void)hipEventDestroy(e0); return e; }
    const size_t n16 = bytes / 16;
    auto launch = [&]() { hipLaunchKernelGGL(copy_kernel, dim3(8192), dim3(256), 0, st, (const v4i *)src, (v4i *)dst, n16); };
    launch();
    (void)hipEventRecord(e0, st);
    for (int i = 0; i < reps; i++) launch();
    (void)hipEventRecord(e1, st);
    e = hipEventSynchronize(e1);
    float ms = 0.0f;
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return e;
    *bytes_per_s = 2.0 * (double)n16 * 16 * reps / (ms * 1e-3);          // read + write
    return hipGetLastError();
}

}  // namespace samp
