// Downstream target on top of the encoder output (Section 3.1, "Downstream Target"): text
// classification on the first token, logits = W_c tanh(W_p h[b, 0] + b_p) + b_c.
// One block per sequence; a wave owns an output channel at a time, its 64 lanes split the hidden
// dimension 8 fp16 weights (16 bytes) per load, binary32 accumulation, wave reduction.  The work is a
// pair of matrix-vector products per sequence (the weights are shared by all blocks through L2).
#include "samp_common.h"

namespace samp {
namespace {

__device__ __forceinline__ float wave_sum_f32(float v)
{
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, 64);
    return v;
}

// dot of one fp16 weight row with the block's vector in LDS
__device__ __forceinline__ float row_dot(const __half *__restrict__ wrow, const float *__restrict__ x, int H, int lane)
{
    float acc = 0.0f;
    for (int k = lane * 8; k < H; k += 512) {
        const v8h w = *reinterpret_cast<const v8h *>(wrow + k);
#pragma unroll
        for (int e = 0; e < 8; e++) acc = __builtin_fmaf((float)w[e], x[k + e], acc);
    }
    return wave_sum_f32(acc);
}

__global__ __launch_bounds__(256) void classify_kernel(const __half *__restrict__ hidden, size_t seq_stride,
                                                       const __half *__restrict__ w_pool, const float *__restrict__ b_pool,
                                                       const __half *__restrict__ w_cls, const float *__restrict__ b_cls,
                                                       int H, int C, float *__restrict__ logits)
{
    extern __shared__ float sm[];                    // h[H], pooled[H]
    float *h = sm, *pooled = sm + H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const __half *src = hidden + (size_t)blockIdx.x * seq_stride;           // first token of the sequence
    for (int k = tid; k < H; k += 256) h[k] = (float)src[k];
    __syncthreads();
    for (int n = wave; n < H; n += 4) {
        const float d = row_dot(w_pool + (size_t)n * H, h, H, lane);
        if (lane == 0) pooled[n] = tanhf(d + b_pool[n]);
    }
    __syncthreads();
    for (int c = wave; c < C; c += 4) {
        const float d = row_dot(w_cls + (size_t)c * H, pooled, H, lane);
        if (lane == 0) logits[(size_t)blockIdx.x * C + c] = d + b_cls[c];
    }
}

}  // namespace

hipError_t launch_classify(const __half *hidden, int B, int S, int H, const __half *w_pool, const float *b_pool,
                           const __half *w_cls, const float *b_cls, int C, float *logits, hipStream_t st)
{
    hipLaunchKernelGGL(classify_kernel, dim3(B), dim3(256), 2 * (size_t)H * sizeof(float), st, hidden, (size_t)S * H, w_pool,
                       b_pool, w_cls, b_cls, H, C, logits);
    return hipGetLastError();
}

}  // namespace samp
