// Softmax attention over packed (padding-free) rows on gfx950 matrix cores.
//
// INT8 flavour (Section 4.2 / Appendix B: the softmax output is quantised with a step fixed at
// calibration, so both batched products are int8 x int8 -> int32):
//     score = float(q.k) * m_sc;  P = softmax(score);  Pq = rne(P / s_p);  ctx = rne(float(Pq.V) * m_ctx)
// Because the step of P is static, P must be fully normalised before it is rounded: a block keeps
// a whole strip of scores on chip (32 queries x all keys of the sequence, <= 512), so the scores
// never touch memory and no running rescale is needed.  Longer sequences take the three-sweep
// kernels further down, which recompute the scores instead of keeping them.
//
// One block = (sequence, head, 32 queries), 4 waves; wave w owns key tiles w, w+4, ... (32 keys
// each).  S^T = K.Q^T is computed so that in the 32x32 MFMA result a lane holds ONE query and 16
// keys: after the softmax those 16 values are, as they stand, the lane's operand of the P.V MFMA.
// Its other operand is V^T, staged per wave through LDS.  Row maxima, row sums and the partial
// P.V products are combined across the 4 waves through LDS (integer partial sums: exact).
// Every floating-point value that decides an int8 code follows one fixed sequence of binary32
// operations; exp and the row sum are evaluated in binary64 and rounded once.
#include "samp_common.h"
#include "mfma_tile.h"

#include <atomic>
#include <hip/hip_ext.h>

namespace samp {
namespace {

constexpr int QB = 32;                 // queries per block
constexpr int ONE_PASS_MAX_LEN = 512;  // longest sequence whose score strip stays in registers
constexpr int VT_STRIDE_I8 = 36;       // bytes per V^T row (32 keys + pad), int8
constexpr int VT_STRIDE_F16 = 72;      // bytes per V^T row (32 keys + pad), fp16

// exp(x) for x <= 0 in binary64: x = k ln2 + r with |r| <= ln2 / 2 (two-part ln2), then
//     exp(r) = 1 + r (1 + r q(r)),
// q a polynomial of degree 8 that interpolates (exp(r) - 1 - r) / r^2 at the nine Chebyshev nodes of
// [-0.34665, 0.34665] (coefficients solved in rational arithmetic and rounded to binary64), scaled by 2^k.
// Checked against a 60-digit exponential with every fused multiply-add emulated exactly: relative error
// below 2^-49 over the whole argument range, far below a binary32 ulp, so rounding the result to binary32
// gives the correctly rounded exponential (up to ties narrower than 2^-49), which is what the quantiser's
// decision is defined on.  One operation shorter than the Taylor polynomial of the same accuracy.
// x must be finite and above -2^30 (the host bounds the score multiplier accordingly): far below -746 the
// scaling by 2^k underflows to 0 like the exponential itself.  The -inf of a masked key is clamped to
// -746 by the caller.  k = rint(x / ln2) comes out of one fma with 1.5 * 2^52: the sum's low dword is k
// as an integer, the sum minus the constant is k as a double.
__device__ __forceinline__ double exp_nonpos(double x)
{
    const double shifted = __builtin_fma(x, 1.44269504088896338700e+00, 6755399441055744.0);
    const int ki = (int)(unsigned)__double_as_longlong(shifted);
    const double k = shifted - 6755399441055744.0;
    double r = __builtin_fma(k, -6.93147180369123816490e-01, x);
    r = __builtin_fma(k, -1.90821492927058770002e-10, r);
    double p = 0x1.28804ab1d4135p-22;
    p = __builtin_fma(p, r, 0x1.72c73b05aa600p-19);
    p = __builtin_fma(p, r, 0x1.a019c99e7c005p-16);
    p = __builtin_fma(p, r, 0x1.a019ad9901febp-13);
    p = __builtin_fma(p, r, 0x1.6c16c17391579p-10);
    p = __builtin_fma(p, r, 0x1.1111111c49a25p-7);
    p = __builtin_fma(p, r, 0x1.5555555554cb5p-5);
    p = __builtin_fma(p, r, 0x1.5555555553b71p-3);
    p = __builtin_fma(p, r, 0.5);
    p = __builtin_fma(p, r, 1.0);
    p = __builtin_fma(p, r, 1.0);
    return __builtin_ldexp(p, ki);
}

// The wave's number inside its block, as a scalar: every test on it (does this wave own key tile j?) then is a
// scalar branch instead of a lane mask with copies of the live registers where the paths join.
__device__ __forceinline__ int wave_index() { return __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6); }

__device__ __forceinline__ int opaque_zero()
{
    int z;
    asm volatile("v_mov_b32 %0, 0" : "=v"(z));
    return z;
}

struct SeqInfo { int t0, n; };
__device__ __forceinline__ SeqInfo seq_info(const int *cu, int b, int max_len)
{
    if (cu) { const int t0 = cu[b]; return {t0, cu[b + 1] - t0}; }
    return {b * max_len, max_len};
}

// PU: the softmax codes are unsigned, rne(P / s_p) in [0, 255] (the variant that spends all 256 codes
//     on [0, 1]).  The matrix core multiplies signed bytes, so it is fed code - 128 (a flip of the top
//     bit) and the missing 128 * sum_k V[k] is added back from a second product of the same V tile with
//     a row of ones; both are exact in int32.
// HIST: also counts every softmax code of a valid (query, key) pair into p_hist[256] (a diagnostic:
//     which of the 256 integers the softmax output uses, as Appendix B tabulates).
// At least two waves per SIMD are asked for so that the register budget is one the matrix-core results fit
// without the accumulation registers: the products then land where the vector ALU reads them.
template <int NT, bool PU, bool HIST>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void attention_i8_kernel(const int8_t *__restrict__ qkv, const int *__restrict__ cu,
                                                           int max_len, int H, float m_sc, float inv_sp, float m_ctx,
                                                           int8_t *__restrict__ ctx, unsigned long long *__restrict__ p_hist)
{
    __shared__ unsigned hist[HIST ? 256 : 1];
    // One slab per wave: first its V^T tiles (written and read by that wave alone), then, once its last P.V
    // product has read them, its partial context for the other waves; sharing the bytes lets a third block fit a CU.
    constexpr int VT_TILE = 64 * VT_STRIDE_I8, SO_BYTES = QB * 64 * 4;
    constexpr int SLAB = NT * VT_TILE > SO_BYTES ? NT * VT_TILE : SO_BYTES;
    __shared__ __attribute__((aligned(16))) int8_t slab[4][SLAB];
    auto so = [&](int wave) { return reinterpret_cast<int(*)[64]>(slab[wave]); };
    __shared__ float smax[4][QB];
    __shared__ double ssum[4][QB];

    // work item = (sequence, head, query block), sequences outermost: XCD x works on the x-th eighth of the
    // sequences, whose tokens it also owns in the kernels before and after this one
    const int nqb = (max_len + QB - 1) / QB, heads = H >> 6;
    const int item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int seq = item / (nqb * heads), head = (item / nqb) % heads;
    const SeqInfo sq = seq_info(cu, seq, max_len);
    const int q0 = (item % nqb) * QB;
    if (q0 >= sq.n) return;
    const int n = sq.n;
    const int tid = threadIdx.x, lane = tid & 63, w = wave_index(), r = lane & 31, g = lane >> 5;
    const unsigned ld = 3u * (unsigned)H;                          // row offsets inside a sequence fit 32 bits
    const int8_t *base = qkv + (size_t)sq.t0 * ld + head * 64;
    if (HIST) hist[tid] = 0;                                      // ordered before its use by the barriers below

    // Q strip: second MFMA operand, lane (query r, half g) holds 16 consecutive bytes of the head dim
    const int qrow = min(q0 + r, n - 1);
    v4i qf[2];
#pragma unroll
    for (int ks = 0; ks < 2; ks++) qf[ks] = *reinterpret_cast<const v4i *>(base + (unsigned)qrow * ld + ks * 32 + g * 16);

    float sc[NT][16];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < NT; i++) {
        const int j0 = (w + 4 * i) * 32;
        if (j0 < n) {                                           // wave-uniform
            // the K rows are requested first, then the V rows: the first product then waits for the K rows only
            const int krow = min(j0 + r, n - 1);
            const int8_t *kp = base + (unsigned)krow * ld + H;
            v4i kf[2];
#pragma unroll
            for (int ks = 0; ks < 2; ks++) kf[ks] = *reinterpret_cast<const v4i *>(kp + ks * 32 + g * 16);
            // stage V^T of this key tile: a lane transposes two 4 keys x 4 channels byte blocks in
            // registers (v_perm_b32) and stores them as dwords of 4 consecutive keys per channel
            const int8_t *vp = base + 2 * H;
            const bool full = j0 + 32 <= n;                      // wave-uniform
            const int cq = lane & 15;
            unsigned d[2][4];                                    // all eight loads are issued before the first is used
            if (full) {                                          // four consecutive key rows: one address, three strides
#pragma unroll
                for (int u = 0; u < 2; u++) {
                    const int8_t *p0 = vp + (unsigned)(j0 + 4 * ((lane >> 4) + 4 * u)) * ld + 4 * cq;
#pragma unroll
                    for (int t = 0; t < 4; t++) d[u][t] = *reinterpret_cast<const unsigned *>(p0 + t * ld);
                }
            } else {
#pragma unroll
                for (int u = 0; u < 2; u++)
#pragma unroll
                    for (int t = 0; t < 4; t++)
                        d[u][t] = *reinterpret_cast<const unsigned *>(vp + (unsigned)min(j0 + 4 * ((lane >> 4) + 4 * u) + t, n - 1) * ld + 4 * cq);
            }
            v16i acc;
#pragma unroll
            for (int e = 0; e < 16; e++) acc[e] = 0;
#pragma unroll
            for (int ks = 0; ks < 2; ks++) acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[ks], qf[ks], acc, 0, 0, 0);
#pragma unroll
            for (int u = 0; u < 2; u++) {
                const int kq = (lane >> 4) + 4 * u;
                const unsigned t01l = __builtin_amdgcn_perm(d[u][1], d[u][0], 0x05010400u), t23l = __builtin_amdgcn_perm(d[u][3], d[u][2], 0x05010400u);
                const unsigned t01h = __builtin_amdgcn_perm(d[u][1], d[u][0], 0x07030602u), t23h = __builtin_amdgcn_perm(d[u][3], d[u][2], 0x07030602u);
                unsigned *dst = reinterpret_cast<unsigned *>(&slab[w][i * VT_TILE + (4 * cq) * VT_STRIDE_I8 + 4 * kq]);
                dst[0 * (VT_STRIDE_I8 / 4)] = __builtin_amdgcn_perm(t23l, t01l, 0x05040100u);
                dst[1 * (VT_STRIDE_I8 / 4)] = __builtin_amdgcn_perm(t23l, t01l, 0x07060302u);
                dst[2 * (VT_STRIDE_I8 / 4)] = __builtin_amdgcn_perm(t23h, t01h, 0x05040100u);
                dst[3 * (VT_STRIDE_I8 / 4)] = __builtin_amdgcn_perm(t23h, t01h, 0x07060302u);
            }
            if (full) {                                          // a full tile needs no masking
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    sc[i][e] = (float)acc[e] * m_sc;
                    mx = __builtin_fmaxf(mx, sc[i][e]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    const int key = j0 + 8 * (e >> 2) + 4 * g + (e & 3);
                    sc[i][e] = key < n ? (float)acc[e] * m_sc : -INFINITY;
                    mx = __builtin_fmaxf(mx, sc[i][e]);
                }
            }
        }                                                        // the scores of a tile past the end are never read
    }
    mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32, 64));
    if (g == 0) smax[w][r] = mx;
    __syncthreads();
    mx = __builtin_fmaxf(__builtin_fmaxf(smax[0][r], smax[1][r]), __builtin_fmaxf(smax[2][r], smax[3][r]));

    // tiles past the end are skipped here and below; only a ragged tile holds masked keys (score -inf), whose
    // argument is clamped so that the exponential comes out as 0; in a full tile every argument is finite
    double part = 0.0;
#pragma unroll
    for (int i = 0; i < NT; i++) {
        const int j0 = (w + 4 * i) * 32;
        if (j0 + 32 <= n) {
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const float ev = (float)exp_nonpos((double)(sc[i][e] - mx));
                sc[i][e] = ev;
                part += (double)ev;
            }
        } else if (j0 < n) {
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const float ev = (float)exp_nonpos((double)__builtin_fmaxf(sc[i][e] - mx, -746.0f));
                sc[i][e] = ev;
                part += (double)ev;
            }
        }
    }
    part += __shfl_xor(part, 32, 64);
    if (g == 0) ssum[w][r] = part;
    __syncthreads();
    const float S = (float)(((ssum[0][r] + ssum[1][r]) + ssum[2][r]) + ssum[3][r]);
    const float rS = __fdiv_rn(1.0f, S);

    // Every accumulator register starts from a zero of its own that the compiler cannot see through: with literal
    // zeros it gives the first product of each path registers of its own and copies all 32 accumulators where the
    // paths join.
    v16i o[2], o1[PU ? 2 : 1];
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
        for (int e = 0; e < 16; e++) { o[cb][e] = opaque_zero(); if (PU) o1[cb][e] = opaque_zero(); }
    const float lo = PU ? 0.0f : -127.0f, hi = PU ? 255.0f : 127.0f;
    const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
#pragma unroll
    for (int i = 0; i < NT; i++) {
        const int j0 = (w + 4 * i) * 32;
        if (j0 < n) {
            v4i pf;
#pragma unroll
            for (int q = 0; q < 4; q++) {
                float f[4];
#pragma unroll
                for (int t = 0; t < 4; t++) {
                    // clamp, then round half to even in the adder: the code is the low byte of f
                    f[t] = __builtin_amdgcn_fmed3f((sc[i][4 * q + t] * rS) * inv_sp, lo, hi) + SAMP_RNE_MAGIC;
                    if (HIST && q0 + r < n && j0 + 8 * q + 4 * g + t < n) atomicAdd(&hist[__float_as_uint(f[t]) & 0xffu], 1u);
                }
                pf[q] = pack_codes(f[0], f[1], f[2], f[3]);
                if (PU) pf[q] ^= (int)0x80808080u;                 // code - 128 as a signed byte
            }
#pragma unroll
            for (int cb = 0; cb < 2; cb++) {
                v4i vf;
#pragma unroll
                for (int q = 0; q < 4; q++)
                    vf[q] = *reinterpret_cast<const int *>(&slab[w][i * VT_TILE + (cb * 32 + r) * VT_STRIDE_I8 + 8 * q + 4 * g]);
                o[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(pf, vf, o[cb], 0, 0, 0);
                if (PU) o1[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ones, vf, o1[cb], 0, 0, 0);
            }
        }
    }
    if (PU) {
#pragma unroll
        for (int cb = 0; cb < 2; cb++)
#pragma unroll
            for (int e = 0; e < 16; e++) o[cb][e] += o1[cb][e] * 128;
    }
    // partial context of this wave: lane holds channel cb*32 + r and queries 8q + 4g + t
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
        for (int e = 0; e < 16; e++) so(w)[8 * (e >> 2) + 4 * g + (e & 3)][cb * 32 + r] = o[cb][e];
    __syncthreads();

    const int query = tid >> 3, c0 = (tid & 7) * 8;
    if (q0 + query < n) {
        int codes[8];
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const int O = ((so(0)[query][c0 + e] + so(1)[query][c0 + e]) + so(2)[query][c0 + e]) + so(3)[query][c0 + e];
            codes[e] = qcode((float)O * m_ctx);
        }
        v2i pk = {pack4(codes[0], codes[1], codes[2], codes[3]), pack4(codes[4], codes[5], codes[6], codes[7])};
        *reinterpret_cast<v2i *>(ctx + (size_t)(sq.t0 + q0 + query) * H + head * 64 + c0) = pk;
    }
    if (HIST && hist[tid]) atomicAdd(&p_hist[tid], (unsigned long long)hist[tid]);   // after the barrier above
}

// ---- QKV GEMM and attention of one (sequence, head) in one kernel ------------------------------------------
// For sequences of at most 128 tokens the QKV tile of one (sequence, head) -- the sequence's token rows times the
// head's 64 query, 64 key and 64 value channels -- is exactly one 128 x 192 block tile of the large-tile GEMM, and it
// is all that head's attention needs (Section 3.2: the QKV GEMM's requantised int8 output is the attention's only
// input).  The block therefore runs that GEMM's main loop (three-deep ring of 64-byte stages, direct global->LDS
// loads, wave tiles of 64 x 96), requantises q, k, v into LDS where the ring was, and goes on as the attention
// kernels above do, one wave per 32 queries over all keys: q, k, v never reach memory and one launch per layer is
// gone.  Every value is produced by the same operations in the same order as in the two separate kernels (row sums
// and, for FP16, partial contexts are accumulated per key tile modulo 4 in ascending order, which is how the four
// waves of those kernels form them), so the context is the same bytes.  QT = 2 is the same for up to 256 tokens: a
// 256 x 192 block tile, wave tiles of 128 x 96, a wave's 64 queries 32 at a time.
template <int QT>                                          // QT 32-query tiles per wave: sequences of at most 128 QT tokens
struct QkvTile {                                           // the block tile both flavours of the kernel share
    static constexpr int TM = 2 * QT, TN = 3, BKB = 64, NSTAGE = 3, NWAVES = 4, CH = 4, RPI = 16, KS = 2;
    static constexpr int BM = 128 * QT, BN = 192;
    static constexpr int A_BYTES = BM * BKB, STAGE_BYTES = (BM + BN) * BKB, RING_BYTES = NSTAGE * STAGE_BYTES;
    static constexpr int NLD = (BM + BN) / RPI / NWAVES;          // 1 KiB pieces per wave and stage
};

// The GEMM part: the wave's (64 QT) x 96 accumulators of X[t0 .. t0+n) . W_head^T, rows of Kbytes bytes; HALF: fp16 operands.
// The main loop of the large-tile GEMM kernel (same ring, same waits); load_tables() runs once the first stages are
// requested.  On return the ring is idle.
// VWAVE: the wave's last two channel tiles are value channels.  Their products are formed with the operands the other
// way round (token rows first), so that a lane of the result holds ONE channel and four consecutive tokens per
// register group: exactly a dword (fp16: 8 bytes) of V^T, which the P.V product wants key-contiguous.  The sums are
// the same (the same products over the same k).  ALL_LIVE: every 32-token tile of the block holds tokens (no tests in
// the loop).
template <int QT, bool HALF, bool VWAVE, bool ALL_LIVE, class Acc, class LoadTables>
__device__ __forceinline__ void qkv_tile_gemm(const char *__restrict__ X, const char *__restrict__ W, int t0, int n, int head, int H,
                                              int Kbytes, char *lds, int wave, int lane, Acc (&acc)[3][2 * QT], LoadTables load_tables)
{
    typedef QkvTile<QT> Tile;
    constexpr int TM = Tile::TM, TN = Tile::TN, BKB = Tile::BKB, NSTAGE = Tile::NSTAGE, NWAVES = Tile::NWAVES;
    constexpr int CH = Tile::CH, RPI = Tile::RPI, KS = Tile::KS, BM = Tile::BM;
    constexpr int A_BYTES = Tile::A_BYTES, STAGE_BYTES = Tile::STAGE_BYTES, RING_BYTES = Tile::RING_BYTES, NLD = Tile::NLD;
    static_assert((Tile::BM + Tile::BN) % (RPI * NWAVES) == 0, "a stage must split into whole pieces per wave");
    const int wm = (wave >> 1) * 32 * TM, wn = (wave & 1) * 32 * TN;
    const int r = lane & 31, g = lane >> 5;
    // operand rows: the sequence's tokens (rows past its end repeat the last one), and the head's 64 rows of each of
    // the query, key and value thirds of the weight matrix
    const char *src[NLD];
#pragma unroll
    for (int j = 0; j < NLD; j++) {
        const int srow = RPI * (wave + NWAVES * j) + lane / CH;
        if (srow < BM) {
            const int am = min(srow, n - 1);
            src[j] = X + (size_t)(t0 + am) * Kbytes + (((lane % CH) ^ swz<BKB>(srow)) << 4);
        } else {
            const int row = srow - BM;
            src[j] = W + (size_t)((row >> 6) * H + head * 64 + (row & 63)) * Kbytes + (((lane % CH) ^ swz<BKB>(row)) << 4);
        }
    }
    const int KT = Kbytes / BKB;
    int fill_slot = 0, fill_kt = 0;
    auto issue = [&]() {
        char *st = lds + fill_slot * STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < NLD; j++)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[j] + (size_t)fill_kt * BKB),
                                             (__attribute__((address_space(3))) void *)(st + (wave + NWAVES * j) * 1024), 16, 0, 0);
        fill_kt++;
        fill_slot = fill_slot + 1 == NSTAGE ? 0 : fill_slot + 1;
    };
    const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) char *)lds;
    unsigned offa[KS], offw[KS];
#pragma unroll
    for (int ks = 0; ks < KS; ks++) {
        offa[ks] = lds_base + (wm + r) * BKB + (((2 * ks + g) ^ swz<BKB>(wm + r)) << 4);
        offw[ks] = lds_base + A_BYTES + (wn + r) * BKB + (((2 * ks + g) ^ swz<BKB>(wn + r)) << 4);
    }
    auto fetch = [&](int slot_bytes, int ks, v4i (&fa)[TM], v4i (&fw)[TN]) {
        lds_read_frags<32 * BKB>(offa[ks] + slot_bytes, fa, std::make_integer_sequence<int, TM>());
        lds_read_frags<32 * BKB>(offw[ks] + slot_bytes, fw, std::make_integer_sequence<int, TN>());
    };
    auto ready = [&](v4i (&fa)[TM], v4i (&fw)[TN]) {
        tie(fa, std::make_integer_sequence<int, TM>());
        tie(fw, std::make_integer_sequence<int, TN>());
    };

#pragma unroll
    for (int s = 0; s < NSTAGE - 1; s++)
        if (s < KT) issue();
    load_tables();

#pragma unroll
    for (int i = 0; i < TN; i++)
#pragma unroll
        for (int j = 0; j < TM; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0;
    bool rows_live[TM];                                           // wave-uniform: token tiles past the sequence's end are not multiplied
#pragma unroll
    for (int j = 0; j < TM; j++) rows_live[j] = wm + 32 * j < n;
    auto multiply = [&](const v4i (&fa)[TM], const v4i (&fw)[TN]) {
#pragma unroll
        for (int j = 0; j < TM; j++)
            if (ALL_LIVE || rows_live[j]) {
#pragma unroll
                for (int i = 0; i < TN; i++) {
                    const bool tokens_first = VWAVE && i >= 1;
                    const v4i first = tokens_first ? fa[j] : fw[i], second = tokens_first ? fw[i] : fa[j];
                    if constexpr (HALF)
                        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_f16(__builtin_bit_cast(v8h, first), __builtin_bit_cast(v8h, second), acc[i][j], 0, 0, 0);
                    else
                        acc[i][j] = __builtin_amdgcn_mfma_i32_32x32x32_i8(first, second, acc[i][j], 0, 0, 0);
                }
            }
    };

    v4i fa[2][TM], fw[2][TN];
    if (KT > NSTAGE - 2) wait_vm_and_barrier<(NSTAGE - 2) * NLD>(); else wait_vm_and_barrier<0>();
    fetch(0, 0, fa[0], fw[0]);
    int slot_bytes = 0;
    auto next_slot = [&]() { slot_bytes = slot_bytes + STAGE_BYTES == RING_BYTES ? 0 : slot_bytes + STAGE_BYTES; };
    auto step = [&](int ks, bool refill, bool more, auto vm_tag) {
        constexpr int VM = decltype(vm_tag)::value;
        if (ks + 1 < KS) {
            fetch(slot_bytes, ks + 1, fa[(ks + 1) & 1], fw[(ks + 1) & 1]);
            wait_lds_reads<TM + TN>();
        } else if (more) {
            wait_vm_and_barrier<VM>();
            next_slot();
            fetch(slot_bytes, 0, fa[0], fw[0]);
        } else {
            wait_lds_reads<0>();
        }
        ready(fa[ks & 1], fw[ks & 1]);
        __builtin_amdgcn_sched_barrier(0);
        if (refill && ks == 0) issue();
        multiply(fa[ks & 1], fw[ks & 1]);
        __builtin_amdgcn_sched_barrier(0);
    };
    int kt = 0;
    for (; kt + NSTAGE - 1 < KT; kt++)
#pragma unroll
        for (int ks = 0; ks < KS; ks++) step(ks, true, true, std::integral_constant<int, (NSTAGE - 2) * NLD>());
    for (; kt + 1 < KT; kt++)
#pragma unroll
        for (int ks = 0; ks < KS; ks++) step(ks, false, true, std::integral_constant<int, 0>());
#pragma unroll
    for (int ks = 0; ks < KS; ks++) step(ks, false, false, std::integral_constant<int, 0>());
    wait_vm_and_barrier<0>();                                     // the ring is idle from here on
}

// one of four copies of the loop: by wave column (value channels or not) and by whether all token tiles are live
template <int QT, bool HALF, class Acc, class LoadTables>
__device__ __forceinline__ void qkv_tile_gemm_any(const char *__restrict__ X, const char *__restrict__ W, int t0, int n, int head, int H,
                                                  int Kbytes, char *lds, int wave, int lane, Acc (&acc)[3][2 * QT], LoadTables load_tables)
{
    const bool all_live = n > QkvTile<QT>::BM - 32;               // block-uniform; wave & 1 is wave-uniform
    if (wave & 1) {
        if (all_live) qkv_tile_gemm<QT, HALF, true, true>(X, W, t0, n, head, H, Kbytes, lds, wave, lane, acc, load_tables);
        else qkv_tile_gemm<QT, HALF, true, false>(X, W, t0, n, head, H, Kbytes, lds, wave, lane, acc, load_tables);
    } else {
        if (all_live) qkv_tile_gemm<QT, HALF, false, true>(X, W, t0, n, head, H, Kbytes, lds, wave, lane, acc, load_tables);
        else qkv_tile_gemm<QT, HALF, false, false>(X, W, t0, n, head, H, Kbytes, lds, wave, lane, acc, load_tables);
    }
}

template <int QT, bool PU>                                 // PU: unsigned softmax codes, as in attention_i8_kernel
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(QT == 1 ? 2 : 1, QT == 1 ? 2 : 1)))
void qkv_attention_i8_kernel(const char *__restrict__ X, const char *__restrict__ W, const float *__restrict__ m_tab,
                             const float *__restrict__ b_tab, const int *__restrict__ cu, int max_len, int H, float m_sc,
                             float inv_sp, float m_ctx, int8_t *__restrict__ ctx)
{
    typedef QkvTile<QT> Tile;
    constexpr int TM = Tile::TM, TN = Tile::TN, BM = Tile::BM, BN = Tile::BN, RING_BYTES = Tile::RING_BYTES, NKT = 4 * QT;
    constexpr int QK_STRIDE = 80, VT_STRIDE = BM + 4;             // bytes per token row of q / k, per channel row of V^T
    constexpr int Q_OFF = 0, K_OFF = BM * QK_STRIDE, VT_OFF = 2 * BM * QK_STRIDE;
    static_assert(VT_OFF + 64 * VT_STRIDE <= RING_BYTES, "q, k and V^T take the place of the ring");
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    float *tab = reinterpret_cast<float *>(lds + RING_BYTES);     // multipliers, then offsets, of the 192 columns

    const int heads = H >> 6;
    const int item = xcd_contiguous(blockIdx.x, gridDim.x);       // sequences outermost, as in the attention kernel
    const int seq = item / heads, head = item % heads;
    const SeqInfo sq = seq_info(cu, seq, max_len);
    const int n = sq.n;
    if (n <= 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
    const int wm = (wave >> 1) * 32 * TM, wn = (wave & 1) * 32 * TN;
    const int r = lane & 31, g = lane >> 5;

    v16i acc[TN][TM];
    qkv_tile_gemm_any<QT, false>(X, W, sq.t0, n, head, H, H, lds, wave, lane, acc, [&]() {
        for (int c = tid; c < BN; c += 256) {
            const int col = (c >> 6) * H + head * 64 + (c & 63);
            tab[c] = m_tab[col];
            tab[BN + c] = b_tab ? b_tab[col] : 0.0f;
        }
    });

    // requantise into LDS: q and k as token rows of 64 codes, v transposed (a channel's codes of all keys in a row).
    // In a query / key tile a lane holds one token and groups of four consecutive channels; in a value tile one channel
    // and groups of four consecutive tokens.
#pragma unroll
    for (int io = 0; io < TN; io++) {
        const int nl = wn + io * 32;                              // first of the tile's 32 columns among the block's 192 (scalar)
        const int part = nl >> 6, c0 = nl & 63;                   // 0 query, 1 key, 2 value
        if (part < 2) {
            v4f mm[4], bb[4];
#pragma unroll
            for (int q = 0; q < 4; q++) {
                mm[q] = *reinterpret_cast<const v4f *>(tab + nl + 8 * q + 4 * g);
                bb[q] = *reinterpret_cast<const v4f *>(tab + BN + nl + 8 * q + 4 * g);
            }
#pragma unroll
            for (int j = 0; j < TM; j++) {
                const int row = wm + 32 * j + r;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const v16i &a = acc[io][j];
                    const int pk = pack_codes(code_bits(__builtin_fmaf((float)a[4 * q + 0], mm[q].x, bb[q].x)),
                                              code_bits(__builtin_fmaf((float)a[4 * q + 1], mm[q].y, bb[q].y)),
                                              code_bits(__builtin_fmaf((float)a[4 * q + 2], mm[q].z, bb[q].z)),
                                              code_bits(__builtin_fmaf((float)a[4 * q + 3], mm[q].w, bb[q].w)));
                    *reinterpret_cast<int *>(lds + (part ? K_OFF : Q_OFF) + row * QK_STRIDE + c0 + 8 * q + 4 * g) = pk;
                }
            }
        } else {
            const float mm = tab[nl + r], bb = tab[BN + nl + r];  // the lane's channel
#pragma unroll
            for (int j = 0; j < TM; j++)
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const v16i &a = acc[io][j];
                    const int pk = pack_codes(code_bits(__builtin_fmaf((float)a[4 * q + 0], mm, bb)), code_bits(__builtin_fmaf((float)a[4 * q + 1], mm, bb)),
                                              code_bits(__builtin_fmaf((float)a[4 * q + 2], mm, bb)), code_bits(__builtin_fmaf((float)a[4 * q + 3], mm, bb)));
                    *reinterpret_cast<int *>(lds + VT_OFF + (c0 + r) * VT_STRIDE + wm + 32 * j + 8 * q + 4 * g) = pk;
                }
        }
    }
    __syncthreads();

    // attention: this wave's 32 QT queries against all keys, 32 queries at a time
#pragma unroll 1
    for (int qt = 0; qt < QT; qt++) {
        const int q0 = (wave * QT + qt) * QB;
        if (q0 >= n) break;                                       // no barrier below
        v4i qf[2];
#pragma unroll
        for (int ks = 0; ks < 2; ks++) qf[ks] = *reinterpret_cast<const v4i *>(lds + Q_OFF + (q0 + r) * QK_STRIDE + ks * 32 + g * 16);
        float sc[NKT][16];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < NKT; i++) {
            const int j0 = 32 * i;
            if (j0 < n) {                                        // wave-uniform
                v4i kf[2];
#pragma unroll
                for (int ks = 0; ks < 2; ks++) kf[ks] = *reinterpret_cast<const v4i *>(lds + K_OFF + (j0 + r) * QK_STRIDE + ks * 32 + g * 16);
                v16i s;
#pragma unroll
                for (int e = 0; e < 16; e++) s[e] = 0;
#pragma unroll
                for (int ks = 0; ks < 2; ks++) s = __builtin_amdgcn_mfma_i32_32x32x32_i8(kf[ks], qf[ks], s, 0, 0, 0);
                if (j0 + 32 <= n) {
#pragma unroll
                    for (int e = 0; e < 16; e++) {
                        sc[i][e] = (float)s[e] * m_sc;
                        mx = __builtin_fmaxf(mx, sc[i][e]);
                    }
                } else {
#pragma unroll
                    for (int e = 0; e < 16; e++) {
                        const int key = j0 + 8 * (e >> 2) + 4 * g + (e & 3);
                        sc[i][e] = key < n ? (float)s[e] * m_sc : -INFINITY;
                        mx = __builtin_fmaxf(mx, sc[i][e]);
                    }
                }
            }
        }
        mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32, 64));

        // row sums: key tile i adds to partial sum i mod 4, in ascending order, as wave i mod 4 of the attention kernel does
        double part[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int i = 0; i < NKT; i++) {
            if (32 * i < n) {                                    // (one copy of the exponentials per tile: the clamp, which only a
#pragma unroll                                                    //  ragged tile needs, costs less than a second copy's instruction fetches)
                for (int e = 0; e < 16; e++) {
                    const float ev = (float)exp_nonpos((double)__builtin_fmaxf(sc[i][e] - mx, -746.0f));
                    sc[i][e] = ev;
                    part[i & 3] += (double)ev;
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 4; u++) part[u] += __shfl_xor(part[u], 32, 64);
        const float S = (float)(((part[0] + part[1]) + part[2]) + part[3]);
        const float rS = __fdiv_rn(1.0f, S);

        v16i o[2], o1[PU ? 2 : 1];
#pragma unroll
        for (int cb = 0; cb < 2; cb++)
#pragma unroll
            for (int e = 0; e < 16; e++) { o[cb][e] = opaque_zero(); if (PU) o1[cb][e] = opaque_zero(); }
        const float lo = PU ? 0.0f : -127.0f, hi = PU ? 255.0f : 127.0f;
        const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
#pragma unroll
        for (int i = 0; i < NKT; i++) {
            const int j0 = 32 * i;
            if (j0 < n) {
                v4i pf;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    float f[4];
#pragma unroll
                    for (int t = 0; t < 4; t++) f[t] = __builtin_amdgcn_fmed3f((sc[i][4 * q + t] * rS) * inv_sp, lo, hi) + SAMP_RNE_MAGIC;
                    pf[q] = pack_codes(f[0], f[1], f[2], f[3]);
                    if (PU) pf[q] ^= (int)0x80808080u;             // code - 128 as a signed byte
                }
#pragma unroll
                for (int cb = 0; cb < 2; cb++) {
                    v4i vf;
#pragma unroll
                    for (int q = 0; q < 4; q++)
                        vf[q] = *reinterpret_cast<const int *>(lds + VT_OFF + (cb * 32 + r) * VT_STRIDE + j0 + 8 * q + 4 * g);
                    o[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf, pf, o[cb], 0, 0, 0);   // channels x queries: a lane holds ONE query
                    if (PU) o1[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(vf, ones, o1[cb], 0, 0, 0);   // 128 times this is added back below
                }
            }
        }

        if (PU) {
#pragma unroll
            for (int cb = 0; cb < 2; cb++)
#pragma unroll
                for (int e = 0; e < 16; e++) o[cb][e] += o1[cb][e] * 128;
        }
        // context codes: the lane's query, channels cb*32 + 8q + 4g + t: four codes per dword into the wave's own query rows
        // in LDS (read into qf above, read by no other wave), from where they leave as 32 bytes per lane
        char *slab = lds + Q_OFF + q0 * QK_STRIDE;
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int cb = 0; cb < 2; cb++)
#pragma unroll
            for (int q = 0; q < 4; q++)
                *reinterpret_cast<int *>(slab + r * QK_STRIDE + cb * 32 + 8 * q + 4 * g) =
                    pack4(qcode((float)o[cb][4 * q] * m_ctx), qcode((float)o[cb][4 * q + 1] * m_ctx), qcode((float)o[cb][4 * q + 2] * m_ctx),
                          qcode((float)o[cb][4 * q + 3] * m_ctx));
        __builtin_amdgcn_wave_barrier();
        const int query = lane >> 1, half = lane & 1;
        if (q0 + query < n) {
            const v4i lo = *reinterpret_cast<const v4i *>(slab + query * QK_STRIDE + half * 32);
            const v4i hi = *reinterpret_cast<const v4i *>(slab + query * QK_STRIDE + half * 32 + 16);
            int8_t *dst = ctx + (size_t)(sq.t0 + q0 + query) * H + head * 64 + half * 32;
            *reinterpret_cast<v4i *>(dst) = lo;
            *reinterpret_cast<v4i *>(dst + 16) = hi;
        }
    }
}

// The FP16 flavour of the kernel above: fp16 QKV GEMM with its bias, q, k, v rounded to fp16 into LDS, then the
// arithmetic of attention_f16_kernel.  The products P.V of the four key tiles are formed from zero one by one and
// added in the order in which that kernel adds its four waves' partial contexts (tiles past the end add +0), and the
// row sums likewise, so the context is the same bytes as from the two kernels.
template <int QT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(QT == 1 ? 2 : 1, QT == 1 ? 2 : 1)))
void qkv_attention_f16_kernel(const char *__restrict__ X, const char *__restrict__ W, const float *__restrict__ bias,
                              const int *__restrict__ cu, int max_len, int H, float scale, __half *__restrict__ ctx)
{
    typedef QkvTile<QT> Tile;
    constexpr int TM = Tile::TM, TN = Tile::TN, BM = Tile::BM, BN = Tile::BN, RING_BYTES = Tile::RING_BYTES, NKT = 4 * QT;
    constexpr int QK_STRIDE = 144, VT_STRIDE = 2 * BM + 8;        // bytes per token row of q / k (64 fp16 + pad), per channel row of V^T (all keys + pad)
    constexpr int Q_OFF = 0, K_OFF = BM * QK_STRIDE, VT_OFF = 2 * BM * QK_STRIDE;
    constexpr int QKV_BYTES = VT_OFF + 64 * VT_STRIDE;            // q, k and V^T take the place of the ring (and more, for 256 tokens)
    constexpr int TAB_OFF = QKV_BYTES > RING_BYTES ? QKV_BYTES : RING_BYTES;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    float *tab = reinterpret_cast<float *>(lds + TAB_OFF);        // bias of the 192 columns

    const int heads = H >> 6;
    const int item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int seq = item / heads, head = item % heads;
    const SeqInfo sq = seq_info(cu, seq, max_len);
    const int n = sq.n;
    if (n <= 0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = wave_index();
    const int wm = (wave >> 1) * 32 * TM, wn = (wave & 1) * 32 * TN;
    const int r = lane & 31, g = lane >> 5;

    v16f acc[TN][TM];
    qkv_tile_gemm_any<QT, true>(X, W, sq.t0, n, head, H, 2 * H, lds, wave, lane, acc, [&]() {
        for (int c = tid; c < BN; c += 256) tab[c] = bias ? bias[(c >> 6) * H + head * 64 + (c & 63)] : 0.0f;
    });

    // fp16(acc + bias) into LDS: q and k as token rows, v transposed (lane layouts as in the INT8 flavour)
#pragma unroll
    for (int io = 0; io < TN; io++) {
        const int nl = wn + io * 32;
        const int part = nl >> 6, c0 = nl & 63;
        if (part < 2) {
            v4f bb[4];
#pragma unroll
            for (int q = 0; q < 4; q++) bb[q] = *reinterpret_cast<const v4f *>(tab + nl + 8 * q + 4 * g);
#pragma unroll
            for (int j = 0; j < TM; j++) {
                const int row = wm + 32 * j + r;
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const v16f &a = acc[io][j];
                    const v4h h = {to_half(a[4 * q] + bb[q].x), to_half(a[4 * q + 1] + bb[q].y), to_half(a[4 * q + 2] + bb[q].z),
                                   to_half(a[4 * q + 3] + bb[q].w)};
                    *reinterpret_cast<v4h *>(lds + (part ? K_OFF : Q_OFF) + row * QK_STRIDE + (c0 + 8 * q + 4 * g) * 2) = h;
                }
            }
        } else {
            const float bb = tab[nl + r];                         // the lane's channel
#pragma unroll
            for (int j = 0; j < TM; j++)
#pragma unroll
                for (int q = 0; q < 4; q++) {
                    const v16f &a = acc[io][j];
                    const v4h h = {to_half(a[4 * q] + bb), to_half(a[4 * q + 1] + bb), to_half(a[4 * q + 2] + bb), to_half(a[4 * q + 3] + bb)};
                    *reinterpret_cast<v4h *>(lds + VT_OFF + (c0 + r) * VT_STRIDE + (wm + 32 * j + 8 * q + 4 * g) * 2) = h;
                }
        }
    }
    __syncthreads();

#pragma unroll 1
    for (int qt = 0; qt < QT; qt++) {
        const int q0 = (wave * QT + qt) * QB;
        if (q0 >= n) break;                                       // no barrier below
        v8h qf[4];
#pragma unroll
        for (int ks = 0; ks < 4; ks++) qf[ks] = *reinterpret_cast<const v8h *>(lds + Q_OFF + (q0 + r) * QK_STRIDE + (ks * 16 + g * 8) * 2);
        float sc[NKT][16];
        float mx = -INFINITY;
#pragma unroll
        for (int i = 0; i < NKT; i++) {
            const int j0 = 32 * i;
            if (j0 < n) {
                v16f s;
#pragma unroll
                for (int e = 0; e < 16; e++) s[e] = 0.0f;
#pragma unroll
                for (int ks = 0; ks < 4; ks++)
                    s = __builtin_amdgcn_mfma_f32_32x32x16_f16(*reinterpret_cast<const v8h *>(lds + K_OFF + (j0 + r) * QK_STRIDE + (ks * 16 + g * 8) * 2),
                                                               qf[ks], s, 0, 0, 0);
#pragma unroll
                for (int e = 0; e < 16; e++) {
                    const int key = j0 + 8 * (e >> 2) + 4 * g + (e & 3);
                    sc[i][e] = key < n ? s[e] * scale : -INFINITY;
                    mx = __builtin_fmaxf(mx, sc[i][e]);
                }
            } else {
#pragma unroll
                for (int e = 0; e < 16; e++) sc[i][e] = -INFINITY;
            }
        }
        mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32, 64));

        float part[4] = {0.0f, 0.0f, 0.0f, 0.0f};                // key tile i adds to partial sum i mod 4, in ascending order
#pragma unroll
        for (int i = 0; i < NKT; i++)
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const float ev = __builtin_amdgcn_exp2f((sc[i][e] - mx) * 1.44269504088896341f);
                sc[i][e] = ev;
                part[i & 3] += ev;
            }
#pragma unroll
        for (int u = 0; u < 4; u++) part[u] += __shfl_xor(part[u], 32, 64);
        const float S = ((part[0] + part[1]) + part[2]) + part[3];
        const float rS = __fdiv_rn(1.0f, S);

        // partial context u: the key tiles u, u + 4, ... from zero, as wave u of the attention kernel forms it; then added in its order
        v16f o[2];
#pragma unroll
        for (int u = 0; u < 4; u++) {
            v16f ot[2];
#pragma unroll
            for (int cb = 0; cb < 2; cb++)
#pragma unroll
                for (int e = 0; e < 16; e++) ot[cb][e] = 0.0f;
#pragma unroll
            for (int ii = 0; ii < QT; ii++) {
                const int i = u + 4 * ii;
                if (32 * i < n) {
#pragma unroll
                    for (int hf = 0; hf < 2; hf++) {                // keys 8q+4g+t for q in {2hf, 2hf+1}
                        v8h pf;
#pragma unroll
                        for (int e = 0; e < 8; e++) pf[e] = to_half(sc[i][8 * hf + e] * rS);
#pragma unroll
                        for (int cb = 0; cb < 2; cb++) {
                            const char *rowp = lds + VT_OFF + (cb * 32 + r) * VT_STRIDE + 32 * i * 2;
                            const v4h lo = *reinterpret_cast<const v4h *>(rowp + (16 * hf + 4 * g) * 2);
                            const v4h hi = *reinterpret_cast<const v4h *>(rowp + (16 * hf + 8 + 4 * g) * 2);
                            const v8h vf = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                            ot[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(vf, pf, ot[cb], 0, 0, 0);   // channels x queries: a lane holds ONE query
                        }
                    }
                }
            }
#pragma unroll
            for (int cb = 0; cb < 2; cb++)
#pragma unroll
                for (int e = 0; e < 16; e++) o[cb][e] = u == 0 ? ot[cb][e] : o[cb][e] + ot[cb][e];
        }

        // context: the lane's query, channels cb*32 + 8q + 4g + t; through the wave's own query rows in LDS, out as 64 bytes per lane
        char *slab = lds + Q_OFF + q0 * QK_STRIDE;
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int cb = 0; cb < 2; cb++)
#pragma unroll
            for (int q = 0; q < 4; q++) {
                const v4h h = {to_half(o[cb][4 * q]), to_half(o[cb][4 * q + 1]), to_half(o[cb][4 * q + 2]), to_half(o[cb][4 * q + 3])};
                *reinterpret_cast<v4h *>(slab + r * QK_STRIDE + (cb * 32 + 8 * q + 4 * g) * 2) = h;
            }
        __builtin_amdgcn_wave_barrier();
        const int query = lane >> 1, half = lane & 1;
        if (q0 + query < n) {
            __half *dst = ctx + (size_t)(sq.t0 + q0 + query) * H + head * 64 + half * 32;
#pragma unroll
            for (int u = 0; u < 4; u++)
                *reinterpret_cast<v4i *>(dst + u * 8) = *reinterpret_cast<const v4i *>(slab + query * QK_STRIDE + half * 64 + u * 16);
        }
    }
}

// FP16 flavour: fp16 q, k, v; binary32 scores, fast exp; P rounded to fp16 before P.V; binary32
// accumulation of P.V.  Optionally records the largest softmax output (calibration of the P step).
template <int NT>
__global__ __launch_bounds__(256) void attention_f16_kernel(const __half *__restrict__ qkv, const int *__restrict__ cu,
                                                            int max_len, int H, float scale, __half *__restrict__ ctx,
                                                            float *__restrict__ p_absmax)
{
    // one slab per wave, as in the INT8 kernel: first its V^T tiles, then its partial context for the other waves
    constexpr int VT_TILE = 64 * VT_STRIDE_F16, SO_BYTES = QB * 64 * 4;
    constexpr int SLAB = NT * VT_TILE > SO_BYTES ? NT * VT_TILE : SO_BYTES;
    __shared__ __attribute__((aligned(16))) char slab[4][SLAB];
    auto so = [&](int wave) { return reinterpret_cast<float(*)[64]>(slab[wave]); };
    __shared__ float smax[4][QB];
    __shared__ float ssum[4][QB];

    // work item = (sequence, head, query block), sequences outermost: XCD x works on the x-th eighth of the
    // sequences, whose tokens it also owns in the kernels before and after this one
    const int nqb = (max_len + QB - 1) / QB, heads = H >> 6;
    const int item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int seq = item / (nqb * heads), head = (item / nqb) % heads;
    const SeqInfo sq = seq_info(cu, seq, max_len);
    const int q0 = (item % nqb) * QB;
    if (q0 >= sq.n) return;
    const int n = sq.n;
    const int tid = threadIdx.x, lane = tid & 63, w = wave_index(), r = lane & 31, g = lane >> 5;
    const unsigned ld = 3u * (unsigned)H;
    const __half *base = qkv + (size_t)sq.t0 * ld + head * 64;

    const int qrow = min(q0 + r, n - 1);
    v8h qf[4];
#pragma unroll
    for (int ks = 0; ks < 4; ks++) qf[ks] = *reinterpret_cast<const v8h *>(base + (unsigned)qrow * ld + ks * 16 + g * 8);

    float sc[NT][16];
    float mx = -INFINITY;
#pragma unroll
    for (int i = 0; i < NT; i++) {
        const int j0 = (w + 4 * i) * 32;
        if (j0 < n) {
            const int krow = min(j0 + r, n - 1);
            const __half *kp = base + (unsigned)krow * ld + H;
            v16f acc;
#pragma unroll
            for (int e = 0; e < 16; e++) acc[e] = 0.0f;
#pragma unroll
            for (int ks = 0; ks < 4; ks++)
                acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(*reinterpret_cast<const v8h *>(kp + ks * 16 + g * 8), qf[ks], acc, 0, 0, 0);
            // stage V^T: lane copies 4 x 8 channels of one key
            const __half *vp = base + 2 * H;
#pragma unroll
            for (int u = 0; u < 4; u++) {
                const int idx = lane + 64 * u, key = idx >> 3, c0 = (idx & 7) * 8;
                const v8h v = *reinterpret_cast<const v8h *>(vp + (unsigned)min(j0 + key, n - 1) * ld + c0);
#pragma unroll
                for (int e = 0; e < 8; e++)
                    *reinterpret_cast<_Float16 *>(&slab[w][i * VT_TILE + (c0 + e) * VT_STRIDE_F16 + key * 2]) = v[e];
            }
#pragma unroll
            for (int e = 0; e < 16; e++) {
                const int key = j0 + 8 * (e >> 2) + 4 * g + (e & 3);
                sc[i][e] = key < n ? acc[e] * scale : -INFINITY;
                mx = __builtin_fmaxf(mx, sc[i][e]);
            }
        } else {
#pragma unroll
            for (int e = 0; e < 16; e++) sc[i][e] = -INFINITY;
        }
    }
    mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32, 64));
    if (g == 0) smax[w][r] = mx;
    __syncthreads();
    mx = __builtin_fmaxf(__builtin_fmaxf(smax[0][r], smax[1][r]), __builtin_fmaxf(smax[2][r], smax[3][r]));

    float part = 0.0f;
#pragma unroll
    for (int i = 0; i < NT; i++)
#pragma unroll
        for (int e = 0; e < 16; e++) {
            const float ev = __builtin_amdgcn_exp2f((sc[i][e] - mx) * 1.44269504088896341f);
            sc[i][e] = ev;
            part += ev;
        }
    part += __shfl_xor(part, 32, 64);
    if (g == 0) ssum[w][r] = part;
    __syncthreads();
    const float S = ((ssum[0][r] + ssum[1][r]) + ssum[2][r]) + ssum[3][r];
    const float rS = __fdiv_rn(1.0f, S);
    if (p_absmax && w == 0 && g == 0 && q0 + r < n)              // the row's largest P is exp(0) / S
        atomicMax(reinterpret_cast<int *>(p_absmax), __float_as_int((float)(_Float16)rS));

    v16f o[2];
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
        for (int e = 0; e < 16; e++) o[cb][e] = 0.0f;
#pragma unroll
    for (int i = 0; i < NT; i++) {
        if ((w + 4 * i) * 32 < n) {
#pragma unroll
            for (int hf = 0; hf < 2; hf++) {                    // keys 8q+4g+t for q in {2hf, 2hf+1}
                v8h pf;
#pragma unroll
                for (int e = 0; e < 8; e++) pf[e] = to_half(sc[i][8 * hf + e] * rS);
#pragma unroll
                for (int cb = 0; cb < 2; cb++) {
                    const char *rowp = &slab[w][i * VT_TILE + (cb * 32 + r) * VT_STRIDE_F16];
                    const v4h lo = *reinterpret_cast<const v4h *>(rowp + (16 * hf + 4 * g) * 2);
                    const v4h hi = *reinterpret_cast<const v4h *>(rowp + (16 * hf + 8 + 4 * g) * 2);
                    const v8h vf = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                    o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(pf, vf, o[cb], 0, 0, 0);
                }
            }
        }
    }
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
        for (int e = 0; e < 16; e++) so(w)[8 * (e >> 2) + 4 * g + (e & 3)][cb * 32 + r] = o[cb][e];
    __syncthreads();

    const int query = tid >> 3, c0 = (tid & 7) * 8;
    if (q0 + query < n) {
        v8h outv;
#pragma unroll
        for (int e = 0; e < 8; e++)
            outv[e] = to_half(((so(0)[query][c0 + e] + so(1)[query][c0 + e]) + so(2)[query][c0 + e]) + so(3)[query][c0 + e]);
        *reinterpret_cast<v8h *>(ctx + (size_t)(sq.t0 + q0 + query) * H + head * 64 + c0) = outv;
    }
}


// ---- sequences longer than 512 keys: the same arithmetic as above, tile by tile ---------------------
// A strip of 32 x n scores no longer fits the registers, so the kernels below sweep the key tiles three
// times: row maxima, row sums, then codes and P.V.  The integer products q.k are recomputed in each
// sweep (two MFMAs per 32 x 32 tile; exact, so all sweeps see the same scores), the exponentials in the
// last two.  A wave still owns key tiles w, w+4, ... and visits them in ascending order, so every
// binary32 / binary64 operation happens in the same order as in the one-pass kernels.

// scores of key tile j0 for the lane's query: sc[e] belongs to key j0 + 8 (e >> 2) + 4 g + (e & 3)
__device__ __forceinline__ void score_tile_i8(const int8_t *base, unsigned ld, int H, int j0, int n, int r, int g,
                                              const v4i (&qf)[2], float m_sc, float (&sc)[16])
{
    const int8_t *kp = base + (unsigned)min(j0 + r, n - 1) * ld + H;
    v16i acc;
#pragma unroll
    for (int e = 0; e < 16; e++) acc[e] = 0;
#pragma unroll
    for (int ks = 0; ks < 2; ks++)
        acc = __builtin_amdgcn_mfma_i32_32x32x32_i8(*reinterpret_cast<const v4i *>(kp + ks * 32 + g * 16), qf[ks], acc, 0, 0, 0);
#pragma unroll
    for (int e = 0; e < 16; e++) {
        const int key = j0 + 8 * (e >> 2) + 4 * g + (e & 3);
        sc[e] = key < n ? (float)acc[e] * m_sc : -INFINITY;
    }
}

template <bool PU, bool HIST>
__global__ __launch_bounds__(256) void attention_i8_long_kernel(const int8_t *__restrict__ qkv, const int *__restrict__ cu,
                                                                int max_len, int H, float m_sc, float inv_sp, float m_ctx,
                                                                int8_t *__restrict__ ctx, unsigned long long *__restrict__ p_hist)
{
    __shared__ unsigned hist[HIST ? 256 : 1];
    __shared__ __attribute__((aligned(16))) int8_t vt[4][64 * VT_STRIDE_I8];
    __shared__ __attribute__((aligned(16))) int so[4][QB][64];
    __shared__ float smax[4][QB];
    __shared__ double ssum[4][QB];

    const int nqb = (max_len + QB - 1) / QB, heads = H >> 6;
    const int item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int seq = item / (nqb * heads), head = (item / nqb) % heads;
    const SeqInfo sq = seq_info(cu, seq, max_len);
    const int q0 = (item % nqb) * QB;
    if (q0 >= sq.n) return;
    const int n = sq.n;
    const int tid = threadIdx.x, lane = tid & 63, w = wave_index(), r = lane & 31, g = lane >> 5;
    const unsigned ld = 3u * (unsigned)H;
    const int8_t *base = qkv + (size_t)sq.t0 * ld + head * 64;
    if (HIST) hist[tid] = 0;

    const int qrow = min(q0 + r, n - 1);
    v4i qf[2];
#pragma unroll
    for (int ks = 0; ks < 2; ks++) qf[ks] = *reinterpret_cast<const v4i *>(base + (unsigned)qrow * ld + ks * 32 + g * 16);

    float sc[16];
    float mx = -INFINITY;
    for (int j0 = w * 32; j0 < n; j0 += 128) {
        score_tile_i8(base, ld, H, j0, n, r, g, qf, m_sc, sc);
#pragma unroll
        for (int e = 0; e < 16; e++) mx = __builtin_fmaxf(mx, sc[e]);
    }
    mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32, 64));
    if (g == 0) smax[w][r] = mx;
    __syncthreads();
    mx = __builtin_fmaxf(__builtin_fmaxf(smax[0][r], smax[1][r]), __builtin_fmaxf(smax[2][r], smax[3][r]));

    double part = 0.0;
    for (int j0 = w * 32; j0 < n; j0 += 128) {
        score_tile_i8(base, ld, H, j0, n, r, g, qf, m_sc, sc);
#pragma unroll
        for (int e = 0; e < 16; e++) part += (double)(float)exp_nonpos((double)__builtin_fmaxf(sc[e] - mx, -746.0f));
    }
    part += __shfl_xor(part, 32, 64);
    if (g == 0) ssum[w][r] = part;
    __syncthreads();
    const float S = (float)(((ssum[0][r] + ssum[1][r]) + ssum[2][r]) + ssum[3][r]);
    const float rS = __fdiv_rn(1.0f, S);

    v16i o[2], o1[PU ? 2 : 1];
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
        for (int e = 0; e < 16; e++) { o[cb][e] = 0; if (PU) o1[cb][e] = 0; }
    const float lo = PU ? 0.0f : -127.0f, hi = PU ? 255.0f : 127.0f;
    const v4i ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    const int8_t *vp = base + 2 * H;
    for (int j0 = w * 32; j0 < n; j0 += 128) {
        score_tile_i8(base, ld, H, j0, n, r, g, qf, m_sc, sc);
        // V^T of this key tile into the wave's own LDS slab (4 keys x 4 channels byte blocks transposed in
        // registers); the slab is written and read by this wave only, in program order
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < 2; u++) {
            const int cq = lane & 15, kq = (lane >> 4) + 4 * u;
            unsigned d[4];
#pragma unroll
            for (int t = 0; t < 4; t++)
                d[t] = *reinterpret_cast<const unsigned *>(vp + (unsigned)min(j0 + 4 * kq + t, n - 1) * ld + 4 * cq);
            const unsigned t01l = __builtin_amdgcn_perm(d[1], d[0], 0x05010400u), t23l = __builtin_amdgcn_perm(d[3], d[2], 0x05010400u);
            const unsigned t01h = __builtin_amdgcn_perm(d[1], d[0], 0x07030602u), t23h = __builtin_amdgcn_perm(d[3], d[2], 0x07030602u);
            unsigned *dst = reinterpret_cast<unsigned *>(&vt[w][(4 * cq) * VT_STRIDE_I8 + 4 * kq]);
            dst[0 * (VT_STRIDE_I8 / 4)] = __builtin_amdgcn_perm(t23l, t01l, 0x05040100u);
            dst[1 * (VT_STRIDE_I8 / 4)] = __builtin_amdgcn_perm(t23l, t01l, 0x07060302u);
            dst[2 * (VT_STRIDE_I8 / 4)] = __builtin_amdgcn_perm(t23h, t01h, 0x05040100u);
            dst[3 * (VT_STRIDE_I8 / 4)] = __builtin_amdgcn_perm(t23h, t01h, 0x07060302u);
        }
        __builtin_amdgcn_wave_barrier();
        v4i pf;
#pragma unroll
        for (int q = 0; q < 4; q++) {
            float f[4];
#pragma unroll
            for (int t = 0; t < 4; t++) {
                const float ev = (float)exp_nonpos((double)__builtin_fmaxf(sc[4 * q + t] - mx, -746.0f));
                f[t] = __builtin_amdgcn_fmed3f((ev * rS) * inv_sp, lo, hi) + SAMP_RNE_MAGIC;
                if (HIST && q0 + r < n && j0 + 8 * q + 4 * g + t < n) atomicAdd(&hist[__float_as_uint(f[t]) & 0xffu], 1u);
            }
            pf[q] = pack_codes(f[0], f[1], f[2], f[3]);
            if (PU) pf[q] ^= (int)0x80808080u;
        }
#pragma unroll
        for (int cb = 0; cb < 2; cb++) {
            v4i vf;
#pragma unroll
            for (int q = 0; q < 4; q++)
                vf[q] = *reinterpret_cast<const int *>(&vt[w][(cb * 32 + r) * VT_STRIDE_I8 + 8 * q + 4 * g]);
            o[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(pf, vf, o[cb], 0, 0, 0);
            if (PU) o1[cb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(ones, vf, o1[cb], 0, 0, 0);
        }
    }
    if (PU) {
#pragma unroll
        for (int cb = 0; cb < 2; cb++)
#pragma unroll
            for (int e = 0; e < 16; e++) o[cb][e] += o1[cb][e] * 128;
    }
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
        for (int e = 0; e < 16; e++) so[w][8 * (e >> 2) + 4 * g + (e & 3)][cb * 32 + r] = o[cb][e];
    __syncthreads();

    const int query = tid >> 3, c0 = (tid & 7) * 8;
    if (q0 + query < n) {
        int codes[8];
#pragma unroll
        for (int e = 0; e < 8; e++) {
            const int O = ((so[0][query][c0 + e] + so[1][query][c0 + e]) + so[2][query][c0 + e]) + so[3][query][c0 + e];
            codes[e] = qcode((float)O * m_ctx);
        }
        v2i pk = {pack4(codes[0], codes[1], codes[2], codes[3]), pack4(codes[4], codes[5], codes[6], codes[7])};
        *reinterpret_cast<v2i *>(ctx + (size_t)(sq.t0 + q0 + query) * H + head * 64 + c0) = pk;
    }
    if (HIST && hist[tid]) atomicAdd(&p_hist[tid], (unsigned long long)hist[tid]);
}

// ---- INT8 attention block whose softmax output stays binary16 (not on the 8-bit grid) ---------------
// P16 = fl16(e * rS), ctx = rne(fl32(sum_k P16[k] V[k]) * m) with m = s_v / s_ctx.  The sum is evaluated
// exactly: a binary16 value in [0, 1] is an integer multiple of 2^-24, so P16 * 2^24 is an integer below
// 2^28 that splits into four 7-bit digits; each digit plane is one more int8 operand for the matrix core
// (non-negative, so no sign trick), the four int32 products recombine in 64-bit integers, and one
// conversion rounds the true sum to binary32.

// V^T of key tile j0 into a wave's own LDS slab: 4 keys x 4 channels byte blocks transposed in registers
__device__ __forceinline__ void stage_vt_i8(const int8_t *vp, unsigned ld, int j0, int n, int lane, int8_t *slab)
{
#pragma unroll
    for (int u = 0; u < 2; u++) {
        const int cq = lane & 15, kq = (lane >> 4) + 4 * u;
        unsigned d[4];
#pragma unroll
        for (int t = 0; t < 4; t++)
            d[t] = *reinterpret_cast<const unsigned *>(vp + (unsigned)min(j0 + 4 * kq + t, n - 1) * ld + 4 * cq);
        const unsigned t01l = __builtin_amdgcn_perm(d[1], d[0], 0x05010400u), t23l = __builtin_amdgcn_perm(d[3], d[2], 0x05010400u);
        const unsigned t01h = __builtin_amdgcn_perm(d[1], d[0], 0x07030602u), t23h = __builtin_amdgcn_perm(d[3], d[2], 0x07030602u);
        unsigned *dst = reinterpret_cast<unsigned *>(&slab[(4 * cq) * VT_STRIDE_I8 + 4 * kq]);
        dst[0 * (VT_STRIDE_I8 / 4)] = __builtin_amdgcn_perm(t23l, t01l, 0x05040100u);
        dst[1 * (VT_STRIDE_I8 / 4)] = __builtin_amdgcn_perm(t23l, t01l, 0x07060302u);
        dst[2 * (VT_STRIDE_I8 / 4)] = __builtin_amdgcn_perm(t23h, t01h, 0x05040100u);
        dst[3 * (VT_STRIDE_I8 / 4)] = __builtin_amdgcn_perm(t23h, t01h, 0x07060302u);
    }
}

// digit planes of one key tile: ev[e] = fl32(exp(score - max)) of the lane's 16 keys; pf[k] is the int8 operand
// holding digit k (7 bits) of P16 * 2^24 for those keys
__device__ __forceinline__ void p16_digits(const float (&ev)[16], float rS, v4i (&pf)[4])
{
#pragma unroll
    for (int q = 0; q < 4; q++) {
        unsigned fixed[4];                                        // P16 * 2^24 of four consecutive keys
#pragma unroll
        for (int t = 0; t < 4; t++) fixed[t] = (unsigned)((float)to_half(ev[4 * q + t] * rS) * 16777216.0f);
#pragma unroll
        for (int k = 0; k < 4; k++)
            pf[k][q] = (int)(((fixed[0] >> (7 * k)) & 127u) | (((fixed[1] >> (7 * k)) & 127u) << 8) |
                             (((fixed[2] >> (7 * k)) & 127u) << 16) | (((fixed[3] >> (7 * k)) & 127u) << 24));
    }
}

// digit planes times the V^T tile in the slab, channel block cb: o[k] += pf[k] . V
__device__ __forceinline__ void p16_mfma(const v4i (&pf)[4], const int8_t *slab, int cb, int r, int g, v16i (&o)[4])
{
    v4i vf;
#pragma unroll
    for (int q = 0; q < 4; q++) vf[q] = *reinterpret_cast<const int *>(&slab[(cb * 32 + r) * VT_STRIDE_I8 + 8 * q + 4 * g]);
#pragma unroll
    for (int k = 0; k < 4; k++) o[k] = __builtin_amdgcn_mfma_i32_32x32x32_i8(pf[k], vf, o[k], 0, 0, 0);
}

// channel block cb: 2^24 times a wave's partial context in 64-bit integers, the four waves added, scaled back
// (exact) and rounded once to binary32.  Contains block-wide barriers.
__device__ __forceinline__ void p16_finish(const v16i (&o)[4], int cb, long long (&so)[4][QB][32], float m_ctx,
                                           int8_t *ctx_rows, int H, int rows_left, int tid)
{
    const int lane = tid & 63, w = wave_index(), r = lane & 31, g = lane >> 5;
    const int query = tid >> 3, c0 = (tid & 7) * 4;
    if (cb) __syncthreads();                                      // the previous block's partials have been read
#pragma unroll
    for (int e = 0; e < 16; e++) {
        const long long v = ((((long long)o[3][e] * 128 + o[2][e]) * 128 + o[1][e]) * 128) + o[0][e];
        so[w][8 * (e >> 2) + 4 * g + (e & 3)][r] = v;
    }
    __syncthreads();
    if (query < rows_left) {
        int codes[4];
#pragma unroll
        for (int e = 0; e < 4; e++) {
            const long long O = ((so[0][query][c0 + e] + so[1][query][c0 + e]) + so[2][query][c0 + e]) + so[3][query][c0 + e];
            const float Of = (float)((double)O * 5.9604644775390625e-08);              // * 2^-24
            codes[e] = qcode(Of * m_ctx);
        }
        *reinterpret_cast<int *>(ctx_rows + (size_t)query * H + cb * 32 + c0) = pack4(codes[0], codes[1], codes[2], codes[3]);
    }
}

// NT > 0: up to 128 NT keys, the strip of scores stays in registers (one pass, as attention_i8_kernel);
// NT == 0: any length, three sweeps (as attention_i8_long_kernel).
template <int NT>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(2))) void
attention_i8_p16_kernel(const int8_t *__restrict__ qkv, const int *__restrict__ cu, int max_len, int H, float m_sc, float m_ctx,
                        int8_t *__restrict__ ctx)
{
    constexpr int NSLAB = NT > 0 ? NT : 1;
    __shared__ __attribute__((aligned(16))) int8_t vt[4][NSLAB][64 * VT_STRIDE_I8];
    __shared__ long long so[4][QB][32];
    __shared__ float smax[4][QB];
    __shared__ double ssum[4][QB];

    const int nqb = (max_len + QB - 1) / QB, heads = H >> 6;
    const int item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int seq = item / (nqb * heads), head = (item / nqb) % heads;
    const SeqInfo sq = seq_info(cu, seq, max_len);
    const int q0 = (item % nqb) * QB;
    if (q0 >= sq.n) return;
    const int n = sq.n;
    const int tid = threadIdx.x, lane = tid & 63, w = wave_index(), r = lane & 31, g = lane >> 5;
    const unsigned ld = 3u * (unsigned)H;
    const int8_t *base = qkv + (size_t)sq.t0 * ld + head * 64;
    const int8_t *vp = base + 2 * H;

    const int qrow = min(q0 + r, n - 1);
    v4i qf[2];
#pragma unroll
    for (int ks = 0; ks < 2; ks++) qf[ks] = *reinterpret_cast<const v4i *>(base + (unsigned)qrow * ld + ks * 32 + g * 16);

    float scr[NSLAB][16];
    float sc[16];
    float mx = -INFINITY;
    if constexpr (NT > 0) {
#pragma unroll
        for (int i = 0; i < NT; i++) {
            const int j0 = (w + 4 * i) * 32;
            if (j0 < n) {
                score_tile_i8(base, ld, H, j0, n, r, g, qf, m_sc, scr[i]);
                stage_vt_i8(vp, ld, j0, n, lane, vt[w][i]);
            } else {
#pragma unroll
                for (int e = 0; e < 16; e++) scr[i][e] = -INFINITY;
            }
#pragma unroll
            for (int e = 0; e < 16; e++) mx = __builtin_fmaxf(mx, scr[i][e]);
        }
    } else {
        for (int j0 = w * 32; j0 < n; j0 += 128) {
            score_tile_i8(base, ld, H, j0, n, r, g, qf, m_sc, sc);
#pragma unroll
            for (int e = 0; e < 16; e++) mx = __builtin_fmaxf(mx, sc[e]);
        }
    }
    mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32, 64));
    if (g == 0) smax[w][r] = mx;
    __syncthreads();
    mx = __builtin_fmaxf(__builtin_fmaxf(smax[0][r], smax[1][r]), __builtin_fmaxf(smax[2][r], smax[3][r]));

    double part = 0.0;
    if constexpr (NT > 0) {
#pragma unroll
        for (int i = 0; i < NT; i++)
#pragma unroll
            for (int e = 0; e < 16; e++) {
                scr[i][e] = (float)exp_nonpos((double)__builtin_fmaxf(scr[i][e] - mx, -746.0f));
                part += (double)scr[i][e];
            }
    } else {
        for (int j0 = w * 32; j0 < n; j0 += 128) {
            score_tile_i8(base, ld, H, j0, n, r, g, qf, m_sc, sc);
#pragma unroll
            for (int e = 0; e < 16; e++) part += (double)(float)exp_nonpos((double)__builtin_fmaxf(sc[e] - mx, -746.0f));
        }
    }
    part += __shfl_xor(part, 32, 64);
    if (g == 0) ssum[w][r] = part;
    __syncthreads();
    const float S = (float)(((ssum[0][r] + ssum[1][r]) + ssum[2][r]) + ssum[3][r]);
    const float rS = __fdiv_rn(1.0f, S);

    int8_t *ctx_rows = ctx + (size_t)(sq.t0 + q0) * H + head * 64;
    if constexpr (NT > 0) {
        // the digit planes of all tiles stay in registers; one channel block at a time halves the accumulators
        v4i pf[NT][4];
#pragma unroll
        for (int i = 0; i < NT; i++) p16_digits(scr[i], rS, pf[i]);
#pragma unroll
        for (int cb = 0; cb < 2; cb++) {
            v16i o[4];
#pragma unroll
            for (int k = 0; k < 4; k++)
#pragma unroll
                for (int e = 0; e < 16; e++) o[k][e] = 0;
#pragma unroll
            for (int i = 0; i < NT; i++)
                if ((w + 4 * i) * 32 < n) p16_mfma(pf[i], vt[w][i], cb, r, g, o);
            p16_finish(o, cb, so, m_ctx, ctx_rows, H, n - q0, tid);
        }
    } else {
        v16i o[2][4];                                         // [channel block][digit plane]
#pragma unroll
        for (int cb = 0; cb < 2; cb++)
#pragma unroll
            for (int k = 0; k < 4; k++)
#pragma unroll
                for (int e = 0; e < 16; e++) o[cb][k][e] = 0;
        for (int j0 = w * 32; j0 < n; j0 += 128) {
            score_tile_i8(base, ld, H, j0, n, r, g, qf, m_sc, sc);
            // the slab is written and read by this wave only, in program order
            __builtin_amdgcn_wave_barrier();
            stage_vt_i8(vp, ld, j0, n, lane, vt[w][0]);
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int e = 0; e < 16; e++) sc[e] = (float)exp_nonpos((double)__builtin_fmaxf(sc[e] - mx, -746.0f));
            v4i pf[4];
            p16_digits(sc, rS, pf);
            p16_mfma(pf, vt[w][0], 0, r, g, o[0]);
            p16_mfma(pf, vt[w][0], 1, r, g, o[1]);
        }
        p16_finish(o[0], 0, so, m_ctx, ctx_rows, H, n - q0, tid);
        p16_finish(o[1], 1, so, m_ctx, ctx_rows, H, n - q0, tid);
    }
}

__device__ __forceinline__ void score_tile_f16(const __half *base, unsigned ld, int H, int j0, int n, int r, int g,
                                               const v8h (&qf)[4], float scale, float (&sc)[16])
{
    const __half *kp = base + (unsigned)min(j0 + r, n - 1) * ld + H;
    v16f acc;
#pragma unroll
    for (int e = 0; e < 16; e++) acc[e] = 0.0f;
#pragma unroll
    for (int ks = 0; ks < 4; ks++)
        acc = __builtin_amdgcn_mfma_f32_32x32x16_f16(*reinterpret_cast<const v8h *>(kp + ks * 16 + g * 8), qf[ks], acc, 0, 0, 0);
#pragma unroll
    for (int e = 0; e < 16; e++) {
        const int key = j0 + 8 * (e >> 2) + 4 * g + (e & 3);
        sc[e] = key < n ? acc[e] * scale : -INFINITY;
    }
}

__global__ __launch_bounds__(256) void attention_f16_long_kernel(const __half *__restrict__ qkv, const int *__restrict__ cu,
                                                                 int max_len, int H, float scale, __half *__restrict__ ctx,
                                                                 float *__restrict__ p_absmax)
{
    __shared__ __attribute__((aligned(16))) char vt[4][64 * VT_STRIDE_F16];
    __shared__ __attribute__((aligned(16))) float so[4][QB][64];
    __shared__ float smax[4][QB];
    __shared__ float ssum[4][QB];

    const int nqb = (max_len + QB - 1) / QB, heads = H >> 6;
    const int item = xcd_contiguous(blockIdx.x, gridDim.x);
    const int seq = item / (nqb * heads), head = (item / nqb) % heads;
    const SeqInfo sq = seq_info(cu, seq, max_len);
    const int q0 = (item % nqb) * QB;
    if (q0 >= sq.n) return;
    const int n = sq.n;
    const int tid = threadIdx.x, lane = tid & 63, w = wave_index(), r = lane & 31, g = lane >> 5;
    const unsigned ld = 3u * (unsigned)H;
    const __half *base = qkv + (size_t)sq.t0 * ld + head * 64;

    const int qrow = min(q0 + r, n - 1);
    v8h qf[4];
#pragma unroll
    for (int ks = 0; ks < 4; ks++) qf[ks] = *reinterpret_cast<const v8h *>(base + (unsigned)qrow * ld + ks * 16 + g * 8);

    float sc[16];
    float mx = -INFINITY;
    for (int j0 = w * 32; j0 < n; j0 += 128) {
        score_tile_f16(base, ld, H, j0, n, r, g, qf, scale, sc);
#pragma unroll
        for (int e = 0; e < 16; e++) mx = __builtin_fmaxf(mx, sc[e]);
    }
    mx = __builtin_fmaxf(mx, __shfl_xor(mx, 32, 64));
    if (g == 0) smax[w][r] = mx;
    __syncthreads();
    mx = __builtin_fmaxf(__builtin_fmaxf(smax[0][r], smax[1][r]), __builtin_fmaxf(smax[2][r], smax[3][r]));

    float part = 0.0f;
    for (int j0 = w * 32; j0 < n; j0 += 128) {
        score_tile_f16(base, ld, H, j0, n, r, g, qf, scale, sc);
#pragma unroll
        for (int e = 0; e < 16; e++) part += __builtin_amdgcn_exp2f((sc[e] - mx) * 1.44269504088896341f);
    }
    part += __shfl_xor(part, 32, 64);
    if (g == 0) ssum[w][r] = part;
    __syncthreads();
    const float S = ((ssum[0][r] + ssum[1][r]) + ssum[2][r]) + ssum[3][r];
    const float rS = __fdiv_rn(1.0f, S);
    if (p_absmax && w == 0 && g == 0 && q0 + r < n)
        atomicMax(reinterpret_cast<int *>(p_absmax), __float_as_int((float)(_Float16)rS));

    v16f o[2];
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
        for (int e = 0; e < 16; e++) o[cb][e] = 0.0f;
    const __half *vp = base + 2 * H;
    for (int j0 = w * 32; j0 < n; j0 += 128) {
        score_tile_f16(base, ld, H, j0, n, r, g, qf, scale, sc);
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int u = 0; u < 4; u++) {
            const int idx = lane + 64 * u, key = idx >> 3, c0 = (idx & 7) * 8;
            const v8h v = *reinterpret_cast<const v8h *>(vp + (unsigned)min(j0 + key, n - 1) * ld + c0);
#pragma unroll
            for (int e = 0; e < 8; e++)
                *reinterpret_cast<_Float16 *>(&vt[w][(c0 + e) * VT_STRIDE_F16 + key * 2]) = v[e];
        }
        __builtin_amdgcn_wave_barrier();
#pragma unroll
        for (int hf = 0; hf < 2; hf++) {
            v8h pf;
#pragma unroll
            for (int e = 0; e < 8; e++)
                pf[e] = to_half(__builtin_amdgcn_exp2f((sc[8 * hf + e] - mx) * 1.44269504088896341f) * rS);
#pragma unroll
            for (int cb = 0; cb < 2; cb++) {
                const char *rowp = &vt[w][(cb * 32 + r) * VT_STRIDE_F16];
                const v4h lo = *reinterpret_cast<const v4h *>(rowp + (16 * hf + 4 * g) * 2);
                const v4h hi = *reinterpret_cast<const v4h *>(rowp + (16 * hf + 8 + 4 * g) * 2);
                const v8h vf = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
                o[cb] = __builtin_amdgcn_mfma_f32_32x32x16_f16(pf, vf, o[cb], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int cb = 0; cb < 2; cb++)
#pragma unroll
        for (int e = 0; e < 16; e++) so[w][8 * (e >> 2) + 4 * g + (e & 3)][cb * 32 + r] = o[cb][e];
    __syncthreads();

    const int query = tid >> 3, c0 = (tid & 7) * 8;
    if (q0 + query < n) {
        v8h outv;
#pragma unroll
        for (int e = 0; e < 8; e++)
            outv[e] = to_half(((so[0][query][c0 + e] + so[1][query][c0 + e]) + so[2][query][c0 + e]) + so[3][query][c0 + e]);
        *reinterpret_cast<v8h *>(ctx + (size_t)(sq.t0 + q0 + query) * H + head * 64 + c0) = outv;
    }
}

}  // namespace

template <bool PU, bool HIST>
static void launch_attention_i8_variant(const int8_t *qkv, const int *cu, int B, int max_len, int H, int heads, float m_sc,
                                        float inv_sp, float m_ctx, int8_t *ctx, unsigned long long *p_hist, hipStream_t st,
                                        const Timing *tm)
{
    dim3 grid((unsigned)((max_len + QB - 1) / QB) * heads * B);
    if (max_len <= 128)
        launch_kernel(attention_i8_kernel<1, PU, HIST>, grid, dim3(256), 0, st, tm, qkv, cu, max_len, H, m_sc, inv_sp, m_ctx, ctx, p_hist);
    else if (max_len <= 256)
        launch_kernel(attention_i8_kernel<2, PU, HIST>, grid, dim3(256), 0, st, tm, qkv, cu, max_len, H, m_sc, inv_sp, m_ctx, ctx, p_hist);
    else if (max_len <= 384)
        launch_kernel(attention_i8_kernel<3, PU, HIST>, grid, dim3(256), 0, st, tm, qkv, cu, max_len, H, m_sc, inv_sp, m_ctx, ctx, p_hist);
    else if (max_len <= ONE_PASS_MAX_LEN)
        launch_kernel(attention_i8_kernel<4, PU, HIST>, grid, dim3(256), 0, st, tm, qkv, cu, max_len, H, m_sc, inv_sp, m_ctx, ctx, p_hist);
    else
        launch_kernel(attention_i8_long_kernel<PU, HIST>, grid, dim3(256), 0, st, tm, qkv, cu, max_len, H, m_sc, inv_sp, m_ctx, ctx, p_hist);
}

hipError_t launch_attention_i8(const int8_t *qkv, const int *cu, int B, int max_len, int H, int heads, float m_sc,
                               float inv_sp, float m_ctx, bool p_unsigned, int8_t *ctx, unsigned long long *p_hist,
                               hipStream_t st, const Timing *tm)
{
    if (p_unsigned) {
        if (p_hist) launch_attention_i8_variant<true, true>(qkv, cu, B, max_len, H, heads, m_sc, inv_sp, m_ctx, ctx, p_hist, st, tm);
        else launch_attention_i8_variant<true, false>(qkv, cu, B, max_len, H, heads, m_sc, inv_sp, m_ctx, ctx, p_hist, st, tm);
    } else {
        if (p_hist) launch_attention_i8_variant<false, true>(qkv, cu, B, max_len, H, heads, m_sc, inv_sp, m_ctx, ctx, p_hist, st, tm);
        else launch_attention_i8_variant<false, false>(qkv, cu, B, max_len, H, heads, m_sc, inv_sp, m_ctx, ctx, p_hist, st, tm);
    }
    return hipGetLastError();
}

template <int QT, bool PU>
static hipError_t launch_qkv_attention_i8_variant(const int8_t *x, const int8_t *w_qkv, const float *m, const float *b, const int *cu,
                                                  int B, int max_len, int H, float m_sc, float inv_sp, float m_ctx, int8_t *ctx,
                                                  hipStream_t st, const Timing *tm)
{
    const size_t lds = QkvTile<QT>::RING_BYTES + 2 * 192 * sizeof(float);
    if (lds > 64 * 1024) {
        static std::atomic<bool> attr_set{false};
        if (!attr_set.load(std::memory_order_acquire)) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(qkv_attention_i8_kernel<QT, PU>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_set.store(true, std::memory_order_release);
        }
    }
    launch_kernel(qkv_attention_i8_kernel<QT, PU>, dim3((unsigned)(B * (H / 64))), dim3(256), lds, st, tm, (const char *)x,
                  (const char *)w_qkv, m, b, cu, max_len, H, m_sc, inv_sp, m_ctx, ctx);
    return hipGetLastError();
}

hipError_t launch_qkv_attention_i8(const int8_t *x, const int8_t *w_qkv, const float *m, const float *b, const int *cu, int B,
                                   int max_len, int H, float m_sc, float inv_sp, float m_ctx, bool p_unsigned, int8_t *ctx,
                                   hipStream_t st, const Timing *tm)
{
    if (max_len > 256 || H % 64 || B <= 0) return hipErrorInvalidValue;
    if (max_len <= 128)
        return p_unsigned ? launch_qkv_attention_i8_variant<1, true>(x, w_qkv, m, b, cu, B, max_len, H, m_sc, inv_sp, m_ctx, ctx, st, tm)
                          : launch_qkv_attention_i8_variant<1, false>(x, w_qkv, m, b, cu, B, max_len, H, m_sc, inv_sp, m_ctx, ctx, st, tm);
    return p_unsigned ? launch_qkv_attention_i8_variant<2, true>(x, w_qkv, m, b, cu, B, max_len, H, m_sc, inv_sp, m_ctx, ctx, st, tm)
                      : launch_qkv_attention_i8_variant<2, false>(x, w_qkv, m, b, cu, B, max_len, H, m_sc, inv_sp, m_ctx, ctx, st, tm);
}

hipError_t launch_qkv_attention_f16(const __half *x, const __half *w_qkv, const float *bias, const int *cu, int B, int max_len,
                                    int H, float scale, __half *ctx, hipStream_t st, const Timing *tm)
{
    if (max_len > 256 || H % 64 || B <= 0) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(B * (H / 64)));
    if (max_len <= 128) {
        const size_t lds = QkvTile<1>::RING_BYTES + 192 * sizeof(float);
        launch_kernel(qkv_attention_f16_kernel<1>, grid, dim3(256), lds, st, tm, (const char *)x, (const char *)w_qkv, bias, cu,
                      max_len, H, scale, ctx);
    } else {
        constexpr size_t qkv_bytes = 2 * 256 * 144 + 64 * (2 * 256 + 8);
        const size_t lds = (qkv_bytes > (size_t)QkvTile<2>::RING_BYTES ? qkv_bytes : (size_t)QkvTile<2>::RING_BYTES) + 192 * sizeof(float);
        static std::atomic<bool> attr_set{false};
        if (!attr_set.load(std::memory_order_acquire)) {
            hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(qkv_attention_f16_kernel<2>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
            if (e != hipSuccess) return e;
            attr_set.store(true, std::memory_order_release);
        }
        launch_kernel(qkv_attention_f16_kernel<2>, grid, dim3(256), lds, st, tm, (const char *)x, (const char *)w_qkv, bias, cu,
                      max_len, H, scale, ctx);
    }
    return hipGetLastError();
}

hipError_t launch_attention_i8_p16(const int8_t *qkv, const int *cu, int B, int max_len, int H, int heads, float m_sc,
                                   float m_ctx, int8_t *ctx, hipStream_t st, const Timing *tm)
{
    dim3 grid((unsigned)((max_len + QB - 1) / QB) * heads * B), block(256);
    if (max_len <= 128) launch_kernel(attention_i8_p16_kernel<1>, grid, block, 0, st, tm, qkv, cu, max_len, H, m_sc, m_ctx, ctx);
    else if (max_len <= 256) launch_kernel(attention_i8_p16_kernel<2>, grid, block, 0, st, tm, qkv, cu, max_len, H, m_sc, m_ctx, ctx);
    else if (max_len <= ONE_PASS_MAX_LEN) launch_kernel(attention_i8_p16_kernel<4>, grid, block, 0, st, tm, qkv, cu, max_len, H, m_sc, m_ctx, ctx);
    else launch_kernel(attention_i8_p16_kernel<0>, grid, block, 0, st, tm, qkv, cu, max_len, H, m_sc, m_ctx, ctx);
    return hipGetLastError();
}

hipError_t launch_attention_f16(const __half *qkv, const int *cu, int B, int max_len, int H, int heads, float scale,
                                __half *ctx, float *p_absmax, hipStream_t st, const Timing *tm)
{
    dim3 grid((unsigned)((max_len + QB - 1) / QB) * heads * B), block(256);
    if (max_len <= 128)
        launch_kernel(attention_f16_kernel<1>, grid, block, 0, st, tm, qkv, cu, max_len, H, scale, ctx, p_absmax);
    else if (max_len <= 256)
        launch_kernel(attention_f16_kernel<2>, grid, block, 0, st, tm, qkv, cu, max_len, H, scale, ctx, p_absmax);
    else if (max_len <= ONE_PASS_MAX_LEN)
        launch_kernel(attention_f16_kernel<4>, grid, block, 0, st, tm, qkv, cu, max_len, H, scale, ctx, p_absmax);
    else
        launch_kernel(attention_f16_long_kernel, grid, block, 0, st, tm, qkv, cu, max_len, H, scale, ctx, p_absmax);
    return hipGetLastError();
}

}  // namespace samp
