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
// A block of 4 waves (2 x 2) computes a (64 TM) x (64 TN) tile, each wave (32 TM) x (32 TN).
// K is consumed 64 bytes per stage through an NSTAGE-deep ring of LDS tiles that is filled by
// direct global->LDS loads (global_load_lds_dwordx4, no register staging), so that NSTAGE-1
// stages of loads are in flight while one is being multiplied: the memory round trip of a step
// is several times longer than its MFMA work, and only a deep ring hides it.  A direct load puts
// lane i's 16 bytes at LDS position i of a 1 KiB run; the XOR swizzle that keeps the operand
// fetches (ds_read_b128) conflict-free is therefore applied to the global address instead.
// Work-groups are renumbered so that each XCD (own L2) owns a contiguous range of tiles.
#include "samp_common.h"
#include "mfma_tile.h"

#include <atomic>
#include <type_traits>
#include <utility>

namespace samp {
namespace {

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

// ---- epilogues -------------------------------------------------------------------------------
// A 32x32 result tile gives each lane 16 accumulators: register 4q+t holds channel
// n_tile + 8q + 4g + t (g = lane >> 5) of the lane's token row.  tile() turns them into the four
// packed output groups of the lane (q = 0..3).  The per-channel tables of the block's BN channels
// are copied into LDS when the block starts (load_tables), so that their memory latency is hidden
// behind the main loop.  load_tab() fetches the table entries of one 32-channel tile from there into registers
// (a Tab) and tile() works from those: the kernels request the Tab of the next tile before they work on the
// current one, because a wave that waits for every LDS read where it needs it spends more time in the
// epilogue of a small problem than in its main loop.
struct EpiRawI32 {                                // test hook: the exact int32 accumulators
    int32_t *out; int N;
    static constexpr int OUT_BYTES = 4;
    static constexpr bool STAGED = false;
    static constexpr int NTAB = 0;
    struct Tab {};
    __device__ __forceinline__ void load_tables(float *, int, int, int, int) const {}
    __device__ __forceinline__ Tab load_tab(const float *, int, int, int) const { return {}; }
    __device__ __forceinline__ void direct(int row, int n, int a0, int a1, int a2, int a3) const
    { *reinterpret_cast<v4i *>(out + (size_t)row * N + n) = v4i{a0, a1, a2, a3}; }
};

__device__ __forceinline__ void copy_table(float *dst, const float *src, int n0, int bn, int tid, int nthreads)
{
    for (int c = tid * 4; c < bn; c += nthreads * 4)
        *reinterpret_cast<v4f *>(dst + c) = src ? *reinterpret_cast<const v4f *>(src + n0 + c) : v4f{0.f, 0.f, 0.f, 0.f};
}

// the multiplier and offset vectors of one 32-channel tile: group q holds channels n_loc + 8q + 4g .. + 3
template <class Tab> __device__ __forceinline__ Tab load_tab_mb(const float *tab, int bn, int n_loc, int g)
{
    Tab t;
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int n = n_loc + 8 * q + 4 * g;
        t.m[q] = *reinterpret_cast<const v4f *>(tab + n);
        t.b[q] = *reinterpret_cast<const v4f *>(tab + bn + n);
    }
    return t;
}

struct EpiRequant {                               // code = rne(fmaf(acc, m[n], b[n]))
    const float *m, *b;
    static constexpr int OUT_BYTES = 1;
    static constexpr bool STAGED = true;
    static constexpr int NTAB = 2;
    typedef int pack_t;
    __device__ __forceinline__ void load_tables(float *tab, int n0, int bn, int tid, int nthreads) const
    { copy_table(tab, m, n0, bn, tid, nthreads); copy_table(tab + bn, b, n0, bn, tid, nthreads); }
    struct Tab { v4f m[4], b[4]; };
    __device__ __forceinline__ Tab load_tab(const float *tab, int bn, int n_loc, int g) const { return load_tab_mb<Tab>(tab, bn, n_loc, g); }
    __device__ __forceinline__ void tile(const v16i &acc, const Tab &t, const float *tab, int bn, int n_loc, int g, int (&pk)[4]) const
    {
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const v4f mm = t.m[q], bb = t.b[q];
            pk[q] = pack_codes(code_bits(__builtin_fmaf((float)acc[4 * q + 0], mm.x, bb.x)),
                               code_bits(__builtin_fmaf((float)acc[4 * q + 1], mm.y, bb.y)),
                               code_bits(__builtin_fmaf((float)acc[4 * q + 2], mm.z, bb.z)),
                               code_bits(__builtin_fmaf((float)acc[4 * q + 3], mm.w, bb.w)));
        }
    }
};

// y = fmaf(acc, m[n], bias[n]); code = rne(GELU(y) / s_out), decided exactly: the fast binary32
// GELU is used wherever it provably rounds like the binary64 definition.  The tie tests leave one
// wave-wide lane mask per accumulator in scalar registers and cost no vector work; only when some
// mask is non-zero (a few percent of the tiles) are they turned into a per-lane bit mask, and the
// flagged elements redone in binary64 by one compact loop (one copy of the slow code per tile).
struct EpiGeluQuant {
    const float *m, *bias; float inv_s;
    static constexpr int OUT_BYTES = 1;
    static constexpr bool STAGED = true;
    static constexpr int NTAB = 2;
    typedef int pack_t;
    __device__ __forceinline__ void load_tables(float *tab, int n0, int bn, int tid, int nthreads) const
    { copy_table(tab, m, n0, bn, tid, nthreads); copy_table(tab + bn, bias, n0, bn, tid, nthreads); }
    struct Tab { v4f m[4], b[4]; };
    __device__ __forceinline__ Tab load_tab(const float *tab, int bn, int n_loc, int g) const { return load_tab_mb<Tab>(tab, bn, n_loc, g); }
    __device__ __forceinline__ void tile(const v16i &acc, const Tab &tb, const float *tab, int bn, int n_loc, int g, int (&pk)[4]) const
    {
        unsigned long long tie[16], any = 0;
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const v4f mm = tb.m[q], bb = tb.b[q];
            float f[4];
#pragma unroll
            for (int t = 0; t < 4; t++) {
                const float y = __builtin_fmaf((float)acc[4 * q + t], mm[t], bb[t]);
                bool near_tie;
                f[t] = gelu_code_bits_fast(y, inv_s, near_tie);
                tie[4 * q + t] = __builtin_amdgcn_ballot_w64(near_tie);
                any |= tie[4 * q + t];
            }
            pk[q] = pack_codes(f[0], f[1], f[2], f[3]);
        }
        if (any == 0) return;                                          // wave-uniform
        const int lane = threadIdx.x & 63;
        unsigned slow = 0;
#pragma unroll
        for (int k = 0; k < 16; k++) slow |= (unsigned)((tie[k] >> lane) & 1) << k;
        while (__builtin_amdgcn_ballot_w64(slow != 0) != 0) {          // wave-uniform loop
            const bool active = slow != 0;
            const int e = active ? __builtin_ctz(slow) : 0;
            int a = acc[0];
#pragma unroll
            for (int k = 1; k < 16; k++) a = (e == k) ? acc[k] : a;
            const int n = n_loc + 8 * (e >> 2) + 4 * g + (e & 3);
            const float y = __builtin_fmaf((float)a, tab[n], tab[bn + n]);
            const int code = qcode(gelu_exact(y) * inv_s);
            const int sh = 8 * (e & 3);
#pragma unroll
            for (int q = 0; q < 4; q++)
                if (active && (e >> 2) == q) pk[q] = (pk[q] & ~(0xff << sh)) | ((code & 0xff) << sh);
            slow &= slow - 1;
        }
    }
};

// The same decision through the threshold table of gelu_table.hip: the bin of y comes out of one fused
// multiply-add (the addend carries 2^23, so the adder rounds to an integer that sits in the low mantissa
// bits), the bin's entry holds the binary32 number at which the code changes inside the bin and the codes
// on either side.  Exact by construction (the table is built from the binary64 definition), about ten
// vector operations and one 8-byte LDS read per element, no transcendental and no slow path.
// The table (at most 16 KiB) is copied into LDS behind the per-channel tables when the block starts.
struct EpiGeluTable {
    const float *m, *bias; const uint32_t *entries; float rate, offset, t_max; int bins;
    static constexpr int OUT_BYTES = 1;
    static constexpr bool STAGED = true;
    static constexpr int NTAB = 2;
    typedef int pack_t;
    __host__ __device__ int extra_lds_bytes() const { return bins * 8; }
    __device__ __forceinline__ void load_tables(float *tab, int n0, int bn, int tid, int nthreads) const
    {
        copy_table(tab, m, n0, bn, tid, nthreads);
        copy_table(tab + bn, bias, n0, bn, tid, nthreads);
        v2i *lut = reinterpret_cast<v2i *>(tab + 2 * bn);
        for (int i = tid; i < bins; i += nthreads) lut[i] = reinterpret_cast<const v2i *>(entries)[i];
    }
    struct Tab { v4f m[4], b[4]; };
    __device__ __forceinline__ Tab load_tab(const float *tab, int bn, int n_loc, int g) const { return load_tab_mb<Tab>(tab, bn, n_loc, g); }
    __device__ __forceinline__ void tile(const v16i &acc, const Tab &t, const float *tab, int bn, int n_loc, int g, int (&pk)[4]) const
    {
        const v2i *lut = reinterpret_cast<const v2i *>(tab + 2 * bn);
        // all sixteen bins first, then the sixteen table reads, then the comparisons: one wait instead of sixteen
        float y[16];
        unsigned bin[16];
        v2i e[16];
#pragma unroll
        for (int k = 0; k < 16; k++) {
            y[k] = __builtin_fmaf((float)acc[k], t.m[k >> 2][k & 3], t.b[k >> 2][k & 3]);
            bin[k] = __float_as_uint(__builtin_amdgcn_fmed3f(__builtin_fmaf(y[k], rate, offset), 8388608.0f, t_max)) - 0x4B000000u;
        }
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < 16; k++) e[k] = lut[bin[k]];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int q = 0; q < 4; q++) {
            unsigned c[4];
#pragma unroll
            for (int k = 0; k < 4; k++)
                c[k] = y[4 * q + k] >= __int_as_float(e[4 * q + k].x) ? (unsigned)e[4 * q + k].y >> 8 : (unsigned)e[4 * q + k].y;
            const unsigned lo = __builtin_amdgcn_perm(c[1], c[0], 0x0c0c0400u), hi = __builtin_amdgcn_perm(c[3], c[2], 0x0c0c0400u);
            pk[q] = (int)__builtin_amdgcn_perm(hi, lo, 0x05040100u);
        }
    }
};

struct EpiF16 {                                   // fp16(act(acc + bias[n]))
    const float *bias; bool gelu;
    static constexpr int OUT_BYTES = 2;
    static constexpr bool STAGED = true;
    static constexpr int NTAB = 1;
    typedef v2i pack_t;
    __device__ __forceinline__ void load_tables(float *tab, int n0, int bn, int tid, int nthreads) const
    { copy_table(tab, bias, n0, bn, tid, nthreads); }
    struct Tab { v4f b[4]; };
    __device__ __forceinline__ Tab load_tab(const float *tab, int bn, int n_loc, int g) const
    {
        Tab t;
#pragma unroll
        for (int q = 0; q < 4; q++) t.b[q] = *reinterpret_cast<const v4f *>(tab + n_loc + 8 * q + 4 * g);
        return t;
    }
    __device__ __forceinline__ void tile(const v16f &acc, const Tab &t, const float *tab, int bn, int n_loc, int g, v2i (&pk)[4]) const
    {
#pragma unroll
        for (int q = 0; q < 4; q++) {
            const v4f bb = t.b[q];
            float a0 = acc[4 * q] + bb.x, a1 = acc[4 * q + 1] + bb.y, a2 = acc[4 * q + 2] + bb.z, a3 = acc[4 * q + 3] + bb.w;
            if (gelu) { a0 = gelu_fast(a0); a1 = gelu_fast(a1); a2 = gelu_fast(a2); a3 = gelu_fast(a3); }
            const v4h h = {to_half(a0), to_half(a1), to_half(a2), to_half(a3)};
            pk[q] = __builtin_bit_cast(v2i, h);
        }
    }
};

template <class Epi> auto extra_lds_of(const Epi &e, int) -> decltype(e.extra_lds_bytes()) { return e.extra_lds_bytes(); }
template <class Epi> int extra_lds_of(const Epi &, long) { return 0; }

// A block is WGM x WGN waves, each computing 32 TM tokens x 32 TN channels.
template <class T, class Epi, int TM, int TN, int BKB, int NSTAGE, int WAVES_PER_EU, int WGM = 2, int WGN = 2>
__global__ __launch_bounds__(64 * WGM * WGN) __attribute__((amdgpu_waves_per_eu(WAVES_PER_EU, 8)))
void gemm_nt_kernel(const char *__restrict__ A, const char *__restrict__ W, char *__restrict__ out, Epi epi, int host_rows,
                    const int *__restrict__ dev_rows, int N, int Kbytes, int tiles_n)
{
    constexpr int NWAVES = WGM * WGN, NT = 64 * NWAVES;
    constexpr int BM = 32 * WGM * TM, BN = 32 * WGN * TN;
    constexpr int A_BYTES = BM * BKB, W_BYTES = BN * BKB, STAGE_BYTES = A_BYTES + W_BYTES;
    constexpr int CH = BKB / 16, RPI = 64 / CH;                  // chunks per row; rows per direct-load instruction
    static_assert(BKB == 64 || BKB == 128, "stage depth");
    static_assert(BM % RPI == 0 && BN % RPI == 0, "operand tiles must be whole 1 KiB pieces");
    // a stage is (BM + BN) / RPI pieces of 1 KiB (the token tile first, then the channel tile), dealt to the
    // waves in turn; when they do not divide evenly the first NPIECE % NWAVES waves issue one load more
    constexpr int NPIECE = (BM + BN) / RPI, NLD = (NPIECE + NWAVES - 1) / NWAVES, NLD_FEWER = NPIECE / NWAVES;
    constexpr int RING_BYTES = NSTAGE * STAGE_BYTES;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    float *tab = reinterpret_cast<float *>(lds + RING_BYTES);

    // each XCD owns a contiguous range of the tiles of the rows that exist (tile order: token rows, then
    // channel tiles), i.e. the same eighth of the token rows as in every other kernel of the path
    const int M = dev_rows ? *dev_rows : host_rows;
    const int tiles = ((M + BM - 1) / BM) * tiles_n;
    if ((int)blockIdx.x >= tiles) return;
    const int tile = xcd_contiguous(blockIdx.x, tiles);
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave / WGN) * 32 * TM, wn = (wave % WGN) * 32 * TN;    // wave tile origin inside the block tile
    const int r = lane & 31, g = lane >> 5;

    // direct loads: instruction j of this wave fills RPI consecutive rows (1 KiB) of an operand tile;
    // lane i supplies row (i / CH), LDS chunk (i % CH), i.e. global chunk (i % CH) ^ swz(row).
    const char *src[NLD];
    const bool fewer = NLD_FEWER != NLD && wave >= NPIECE % NWAVES;   // this wave has no last piece
#pragma unroll
    for (int j = 0; j < NLD; j++) {
        const int piece = min(wave + NWAVES * j, NPIECE - 1);
        const int srow = RPI * piece + lane / CH;                // row inside the stage
        if (srow < BM) {
            int am = m0 + srow; if (am > M - 1) am = M - 1;      // rows past the end re-read the last row
            src[j] = A + (size_t)am * Kbytes + (((lane % CH) ^ swz<BKB>(srow)) << 4);
        } else {
            const int row = srow - BM;
            src[j] = W + (size_t)(n0 + row) * Kbytes + (((lane % CH) ^ swz<BKB>(row)) << 4);
        }
    }
    auto issue = [&](int kt) {
        char *st = lds + (kt % NSTAGE) * STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < NLD; j++)
            if (j < NLD_FEWER || !fewer)
                __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[j] + (size_t)kt * BKB),
                                                 (__attribute__((address_space(3))) void *)(st + (wave + NWAVES * j) * 1024), 16, 0, 0);
    };
    // stage kt has landed when at most the loads of the (NSTAGE - 2) later stages are outstanding
    auto wait_stage = [&](bool later_stages_in_flight) {
        if (!later_stages_in_flight) wait_vm_and_barrier<0>();
        else if (fewer) wait_vm_and_barrier<(NSTAGE - 2) * NLD_FEWER>();
        else wait_vm_and_barrier<(NSTAGE - 2) * NLD>();
    };

    const int KT = Kbytes / BKB;
#pragma unroll
    for (int s = 0; s < NSTAGE - 1; s++)
        if (s < KT) issue(s);
    epi.load_tables(tab, n0, BN, tid, NT);            // ordinary loads; consumed after the main loop

    typename T::acc_t acc[TN][TM];                                // [channel tile][token tile]
#pragma unroll
    for (int i = 0; i < TN; i++)
#pragma unroll
        for (int j = 0; j < TM; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0;

    for (int kt = 0; kt < KT; kt++) {
        // stage kt must have landed: all but the loads of the (up to NSTAGE-2) later stages
        wait_stage(kt + NSTAGE - 2 < KT);
        if (kt + NSTAGE - 1 < KT) issue(kt + NSTAGE - 1);        // refills the buffer consumed at kt-1
        const char *cur = lds + (kt % NSTAGE) * STAGE_BYTES;
#pragma unroll
        for (int ks = 0; ks < CH / 2; ks++) {
            v4i fa[TM], fw[TN];
#pragma unroll
            for (int j = 0; j < TM; j++) {
                const int row = wm + j * 32 + r;
                fa[j] = *reinterpret_cast<const v4i *>(cur + row * BKB + (((2 * ks + g) ^ swz<BKB>(row)) << 4));
            }
#pragma unroll
            for (int i = 0; i < TN; i++) {
                const int row = wn + i * 32 + r;
                fw[i] = *reinterpret_cast<const v4i *>(cur + A_BYTES + row * BKB + (((2 * ks + g) ^ swz<BKB>(row)) << 4));
            }
#pragma unroll
            for (int i = 0; i < TN; i++)
#pragma unroll
                for (int j = 0; j < TM; j++) acc[i][j] = T::mma(fw[i], fa[j], acc[i][j]);
        }
    }
    typename Epi::Tab tabs[TN];                                   // the epilogue's table entries arrive while the waves gather
#pragma unroll
    for (int io = 0; io < TN; io++) tabs[io] = epi.load_tab(tab, BN, wn + io * 32, g);
    wait_vm_and_barrier<0>();                                     // the ring is idle from here on

    if constexpr (!Epi::STAGED) {
#pragma unroll
        for (int io = 0; io < TN; io++)
#pragma unroll
            for (int j = 0; j < TM; j++) {
                const int row = m0 + wm + j * 32 + r;
                if (row < M) {
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const int n = n0 + wn + io * 32 + 8 * q + 4 * g;
                        epi.direct(row, n, acc[io][j][4 * q], acc[io][j][4 * q + 1], acc[io][j][4 * q + 2], acc[io][j][4 * q + 3]);
                    }
                }
            }
    } else {
        // stage the output tile in LDS, then write full rows, 16 bytes per lane
        constexpr int OB = Epi::OUT_BYTES;
        constexpr int STRIDE = BN * OB + 16;
        static_assert(BM * STRIDE <= RING_BYTES, "staging tile does not fit in the ring");
#pragma unroll
        for (int io = 0; io < TN; io++)
#pragma unroll
            for (int j = 0; j < TM; j++) {
                typename Epi::pack_t pk[4];
                const int lrow = wm + j * 32 + r;
                const int nl = wn + io * 32;
                epi.tile(acc[io][j], tabs[io], tab, BN, nl, g, pk);
#pragma unroll
                for (int q = 0; q < 4; q++)
                    *reinterpret_cast<typename Epi::pack_t *>(lds + lrow * STRIDE + (nl + 8 * q + 4 * g) * OB) = pk[q];
            }
        __syncthreads();
        constexpr int CHUNKS = BN * OB / 16;                      // 16-byte chunks per output row
        static_assert((BM * CHUNKS) % NT == 0, "output chunks must split evenly over the threads");
#pragma unroll
        for (int p = 0; p < BM * CHUNKS / NT; p++) {
            const int idx = p * NT + tid;
            const int lrow = idx / CHUNKS, ochunk = idx % CHUNKS;
            if (m0 + lrow < M) {
                const v4i v = *reinterpret_cast<const v4i *>(lds + lrow * STRIDE + ochunk * 16);
                *reinterpret_cast<v4i *>(out + ((size_t)(m0 + lrow) * N + n0) * OB + ochunk * 16) = v;
            }
        }
    }
}

template <class T, class Epi, int TM, int TN, int BKB, int NSTAGE, int WPE, int WGM = 2, int WGN = 2>
hipError_t launch_cfg(const void *A, const void *W, void *out, const Epi &epi, Rows rows, int N, int K, hipStream_t st,
                      const Timing *tm)
{
    constexpr int BM = 32 * WGM * TM, BN = 32 * WGN * TN;
    constexpr size_t LDS_FIXED = (size_t)NSTAGE * (BM + BN) * BKB + (size_t)Epi::NTAB * BN * sizeof(float);
    const size_t LDS = LDS_FIXED + extra_lds_of(epi, 0);
    if (N % BN) return hipErrorInvalidValue;
    if ((K * T::ELEM) % BKB) return hipErrorInvalidValue;
    auto kern = gemm_nt_kernel<T, Epi, TM, TN, BKB, NSTAGE, WPE, WGM, WGN>;
    // > 64 KiB of dynamic LDS must be enabled once per kernel (for the largest table an epilogue may bring);
    // setting it twice from two threads is harmless
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                           (int)(LDS_FIXED + GELU_TABLE_MAX_BINS * 8));
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    const int tiles_n = N / BN, tiles_m = (rows.host_rows + BM - 1) / BM, total = tiles_n * tiles_m;
    launch_kernel(kern, dim3(total), dim3(64 * WGM * WGN), LDS, st, tm,
                          (const char *)A, (const char *)W, (char *)out, epi, rows.host_rows, rows.dev_rows, N, K * T::ELEM,
                          tiles_n);
    return hipGetLastError();
}


// ---- large tiles ---------------------------------------------------------------------------------
// For many tokens the block tile grows to (64 TM) x (64 TN) with wave tiles of (32 TM) x (32 TN), up to
// 256 x 256 with 128 x 128 per wave: a 32 x 32 x 32 MFMA takes 32 clocks and eats 2 KiB of LDS operands,
// so a wave tile of TM x TN such products needs (TM + TN) / (TM TN) KiB per 32 clocks -- with 2 x 2 the
// four SIMDs of a CU ask for the whole LDS bandwidth, with 4 x 4 for half of it -- and a block tile of
// BM x BN pulls (BM + BN) bytes per BM BN multiply-adds out of L2.  One wave per SIMD, so the latencies
// are hidden by software pipelining instead of by other waves: the K stages (64 bytes) travel through
// an NSTAGE-deep ring of direct global->LDS loads, and the operand fragments of the next 32-byte step
// are fetched from LDS into a second register set while the MFMAs of the current one run.
template <class T, class Epi, int TM, int TN, int BKB, int NSTAGE, int WPE>
__global__ __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(WPE, WPE)))
void gemm_nt_big_kernel(const char *__restrict__ A, const char *__restrict__ W, char *__restrict__ out, Epi epi, int host_rows,
                        const int *__restrict__ dev_rows, int N, int Kbytes, int tiles_n)
{
    constexpr int CH = BKB / 16, RPI = 64 / CH, KS = BKB / 32, NWAVES = 4, NT = 256;
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr int A_BYTES = BM * BKB, STAGE_BYTES = (BM + BN) * BKB;
    constexpr int NLD = (BM + BN) / RPI / NWAVES;                 // 1 KiB pieces per wave and stage
    constexpr int RING_BYTES = NSTAGE * STAGE_BYTES;
    static_assert(BKB == 64 || BKB == 128, "stage depth");
    static_assert(NSTAGE >= 2, "the ring must hold the stage in use and one in flight");
    static_assert((BM + BN) % (RPI * NWAVES) == 0, "a stage must split into whole pieces per wave");
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    float *tab = reinterpret_cast<float *>(lds + RING_BYTES);

    const int M = dev_rows ? *dev_rows : host_rows;
    const int tiles = ((M + BM - 1) / BM) * tiles_n;
    if ((int)blockIdx.x >= tiles) return;
    const int tile = xcd_contiguous(blockIdx.x, tiles);
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave >> 1) * 32 * TM, wn = (wave & 1) * 32 * TN;
    const int r = lane & 31, g = lane >> 5;

    const char *src[NLD];
#pragma unroll
    for (int j = 0; j < NLD; j++) {
        const int srow = RPI * (wave + NWAVES * j) + lane / CH;
        if (srow < BM) {
            int am = m0 + srow; if (am > M - 1) am = M - 1;
            src[j] = A + (size_t)am * Kbytes + (((lane % CH) ^ swz<BKB>(srow)) << 4);
        } else {
            const int row = srow - BM;
            src[j] = W + (size_t)(n0 + row) * Kbytes + (((lane % CH) ^ swz<BKB>(row)) << 4);
        }
    }
    const int KT = Kbytes / BKB;
    int fill_slot = 0, fill_kt = 0;                               // next stage to request and the ring slot it goes to
    auto issue = [&]() {
        char *st = lds + fill_slot * STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < NLD; j++)
            __builtin_amdgcn_global_load_lds((const __attribute__((address_space(1))) void *)(src[j] + (size_t)fill_kt * BKB),
                                             (__attribute__((address_space(3))) void *)(st + (wave + NWAVES * j) * 1024), 16, 0, 0);
        fill_kt++;
        fill_slot = fill_slot + 1 == NSTAGE ? 0 : fill_slot + 1;
    };
    // LDS address of this lane's first fragment of either operand inside a stage, for each 32-byte step of a
    // stage; the fragments of the other 32-row tiles of the wave lie whole multiples of 32 rows further on (the
    // swizzle only looks at row bits 0..3)
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
    epi.load_tables(tab, n0, BN, tid, NT);

    typename T::acc_t acc[TN][TM];
#pragma unroll
    for (int i = 0; i < TN; i++)
#pragma unroll
        for (int j = 0; j < TM; j++)
#pragma unroll
            for (int e = 0; e < 16; e++) acc[i][j][e] = 0;
    auto multiply = [&](const v4i (&fa)[TM], const v4i (&fw)[TN]) {
#pragma unroll
        for (int i = 0; i < TN; i++)
#pragma unroll
            for (int j = 0; j < TM; j++) acc[i][j] = T::mma(fw[i], fa[j], acc[i][j]);
    };

    v4i fa[2][TM], fw[2][TN];                                     // fragments of the current and of the next 32-byte step
    // stage 0 has landed when only the later prologue stages are outstanding
    if (KT > NSTAGE - 2) wait_vm_and_barrier<(NSTAGE - 2) * NLD>(); else wait_vm_and_barrier<0>();
    fetch(0, 0, fa[0], fw[0]);
    // One iteration per stage.  Its first step refills the ring slot that was read last in the iteration before
    // (that iteration's barrier lies between); every step first requests the fragments of the step after it --
    // the last one from the next stage, after waiting for that stage -- then waits for its own fragments only
    // (requested a step ago: the TM + TN requests just made stay outstanding) and multiplies.  The scheduling
    // fences keep the steps apart.  Three copies of the body (stages that still refill the ring, stages that
    // only drain it, the last stage) keep every wait count a constant.
    int slot_bytes = 0;
    auto next_slot = [&]() { slot_bytes = slot_bytes + STAGE_BYTES == RING_BYTES ? 0 : slot_bytes + STAGE_BYTES; };
    auto step = [&](int ks, bool refill, bool more, auto vm_tag) {
        constexpr int VM = decltype(vm_tag)::value;
        if (ks + 1 < KS) {
            fetch(slot_bytes, ks + 1, fa[(ks + 1) & 1], fw[(ks + 1) & 1]);
            wait_lds_reads<TM + TN>();
        } else if (more) {
            wait_vm_and_barrier<VM>();                            // own fragments too (lgkmcnt 0): the slot may be refilled after this
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
    typename Epi::Tab first_tab = epi.load_tab(tab, BN, wn, g);    // arrives while the waves gather
    wait_vm_and_barrier<0>();                                     // the ring is idle from here on

    if constexpr (!Epi::STAGED) {
#pragma unroll
        for (int io = 0; io < TN; io++)
#pragma unroll
            for (int j = 0; j < TM; j++) {
                const int row = m0 + wm + j * 32 + r;
                if (row < M) {
#pragma unroll
                    for (int q = 0; q < 4; q++) {
                        const int n = n0 + wn + io * 32 + 8 * q + 4 * g;
                        epi.direct(row, n, acc[io][j][4 * q], acc[io][j][4 * q + 1], acc[io][j][4 * q + 2], acc[io][j][4 * q + 3]);
                    }
                }
            }
    } else {
        // the output tile goes through LDS 64 token rows at a time (32 of each wave row), then out as full rows
        constexpr int OB = Epi::OUT_BYTES;
        constexpr int STRIDE = BN * OB + 16;
        constexpr int CHUNKS = BN * OB / 16;
        static_assert(2 * 64 * STRIDE <= RING_BYTES, "two staging slabs must fit in the ring");
        static_assert((64 * CHUNKS) % NT == 0, "output chunks must split evenly over the threads");
#pragma unroll
        for (int j = 0; j < TM; j++) {
            char *slab = lds + (j & 1) * 64 * STRIDE;             // alternate slabs: one barrier per pass
            const int lrow = (wave >> 1) * 32 + r;
            typename Epi::Tab cur = j == 0 ? first_tab : epi.load_tab(tab, BN, wn, g);
#pragma unroll
            for (int io = 0; io < TN; io++) {
                typename Epi::pack_t pk[4];
                const int nl = wn + io * 32;
                typename Epi::Tab nxt;                            // the next tile's entries travel while this tile is worked on
                if (io + 1 < TN) nxt = epi.load_tab(tab, BN, nl + 32, g);
                __builtin_amdgcn_sched_barrier(0);
                epi.tile(acc[io][j], cur, tab, BN, nl, g, pk);
#pragma unroll
                for (int q = 0; q < 4; q++)
                    *reinterpret_cast<typename Epi::pack_t *>(slab + lrow * STRIDE + (nl + 8 * q + 4 * g) * OB) = pk[q];
                if (io + 1 < TN) cur = nxt;
            }
            __syncthreads();
            constexpr int PASSES = 64 * CHUNKS / NT;
            v4i v[PASSES];                                        // all reads of the pass, then the stores
#pragma unroll
            for (int p = 0; p < PASSES; p++) {
                const int idx = p * NT + tid;
                v[p] = *reinterpret_cast<const v4i *>(slab + (idx / CHUNKS) * STRIDE + (idx % CHUNKS) * 16);
            }
#pragma unroll
            for (int p = 0; p < PASSES; p++) {
                const int idx = p * NT + tid;
                const int srow = idx / CHUNKS, ochunk = idx % CHUNKS;
                const int grow = m0 + (srow >> 5) * 32 * TM + j * 32 + (srow & 31);
                if (grow < M) *reinterpret_cast<v4i *>(out + ((size_t)grow * N + n0) * OB + ochunk * 16) = v[p];
            }
        }
    }
}

template <class T, class Epi, int TM, int TN, int BKB, int NSTAGE, int WPE = 1>
hipError_t launch_big(const void *A, const void *W, void *out, const Epi &epi, Rows rows, int N, int K, hipStream_t st,
                      const Timing *tm)
{
    constexpr int BM = 64 * TM, BN = 64 * TN;
    constexpr size_t LDS_FIXED = (size_t)NSTAGE * (BM + BN) * BKB + (size_t)Epi::NTAB * BN * sizeof(float);
    const size_t LDS = LDS_FIXED + extra_lds_of(epi, 0);
    if (N % BN || (K * T::ELEM) % BKB || LDS > 160 * 1024) return hipErrorInvalidValue;
    auto kern = gemm_nt_big_kernel<T, Epi, TM, TN, BKB, NSTAGE, WPE>;
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        const size_t cap = std::min<size_t>(LDS_FIXED + GELU_TABLE_MAX_BINS * 8, 160 * 1024);
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize, (int)cap);
        if (e != hipSuccess) return e;
        attr_set.store(true, std::memory_order_release);
    }
    const int tiles_n = N / BN, tiles_m = (rows.host_rows + BM - 1) / BM;
    launch_kernel(kern, dim3(tiles_n * tiles_m), dim3(256), LDS, st, tm,
                  (const char *)A, (const char *)W, (char *)out, epi, rows.host_rows, rows.dev_rows, N, K * T::ELEM, tiles_n);
    return hipGetLastError();
}


// ---- long operand rows on few tiles ------------------------------------------------------------------
// FFN2 at small batch: 24 (FP16: 48) stages of 128 bytes, 64 x 96 tiles that no more than fill the chip once.  Such
// a block is a chain of dependent stages whose pace is set by bytes in flight over load latency, and LDS for a
// deeper ring is what the other batch group's kernels on the same CU need.  Here the stages in flight wait in
// REGISTERS instead (a 32 x 32 tile per wave leaves most of them idle): every wave keeps DEPTH stages of its share
// of the loads outstanding, writes the oldest one to one of two LDS buffers when it lands, and requests the stage
// DEPTH ahead into the registers just freed.  One barrier per stage: a buffer is rewritten two stages after it
// was read, and the barrier of the stage between lies between.  Deeper is faster for the kernel alone and slower
// for the forward (the loads in flight compete with the other group's kernels), so the launcher takes DEPTH = 2:
// what is won is the LDS (40 KB against 61 KB for the three-deep ring).
template <class T, class Epi, int WGN, int DEPTH>
__global__ __launch_bounds__(128 * WGN)
void gemm_nt_longk_kernel(const char *__restrict__ A, const char *__restrict__ W, char *__restrict__ out, Epi epi, int host_rows,
                          const int *__restrict__ dev_rows, int N, int Kbytes, int tiles_n)
{
    constexpr int BKB = 128, BM = 64, BN = 32 * WGN, NWAVES = 2 * WGN, NT = 64 * NWAVES;
    constexpr int NPIECE = (BM + BN) / 8, NLD = (NPIECE + NWAVES - 1) / NWAVES;      // 1 KiB pieces of 8 rows; loads per wave and stage
    constexpr int STAGE_BYTES = (BM + BN) * BKB, A_BYTES = BM * BKB;
    extern __shared__ __attribute__((aligned(1024))) char lds[];
    float *tab = reinterpret_cast<float *>(lds + 2 * STAGE_BYTES);

    const int M = dev_rows ? *dev_rows : host_rows;
    const int tiles = ((M + BM - 1) / BM) * tiles_n;
    if ((int)blockIdx.x >= tiles) return;
    const int tile = xcd_contiguous(blockIdx.x, tiles);
    const int m0 = (tile / tiles_n) * BM, n0 = (tile % tiles_n) * BN;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wm = (wave / WGN) * 32, wn = (wave % WGN) * 32;
    const int r = lane & 31, g = lane >> 5;

    // this wave's pieces: where they come from and where they go (a surplus slot repeats the last piece)
    const char *src[NLD];
    int dst[NLD];
#pragma unroll
    for (int j = 0; j < NLD; j++) {
        const int piece = min(wave + NWAVES * j, NPIECE - 1);
        const int srow = 8 * piece + (lane >> 3), chunk = lane & 7;
        if (srow < BM) {
            int am = m0 + srow; if (am > M - 1) am = M - 1;
            src[j] = A + (size_t)am * Kbytes + chunk * 16;
            dst[j] = srow * BKB + ((chunk ^ swz<BKB>(srow)) << 4);
        } else {
            const int row = srow - BM;
            src[j] = W + (size_t)(n0 + row) * Kbytes + chunk * 16;
            dst[j] = A_BYTES + row * BKB + ((chunk ^ swz<BKB>(row)) << 4);
        }
    }
    const int KT = Kbytes / BKB;                                  // a multiple of DEPTH (the launcher checks)
    // (scheduling fences keep the loads in stage order: the wait for a stage's registers counts the loads behind it)
    v4i held[DEPTH][NLD];
    epi.load_tables(tab, n0, BN, tid, NT);
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int d = 0; d < DEPTH; d++) {
#pragma unroll
        for (int j = 0; j < NLD; j++) held[d][j] = *reinterpret_cast<const v4i *>(src[j] + (size_t)d * BKB);
        __builtin_amdgcn_sched_barrier(0);
    }

    typename T::acc_t acc;
#pragma unroll
    for (int e = 0; e < 16; e++) acc[e] = 0;
    const int offa = (wm + r) * BKB, offw = A_BYTES + (wn + r) * BKB;
    const int sa = swz<BKB>(wm + r), sw = swz<BKB>(wn + r);

    auto stage = [&](int kt, int d, bool refill) {
        char *buf = lds + (kt & 1) * STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < NLD; j++) *reinterpret_cast<v4i *>(buf + dst[j]) = held[d][j];    // waits for these loads only
        __builtin_amdgcn_sched_barrier(0);
        if (refill) {
#pragma unroll
            for (int j = 0; j < NLD; j++) held[d][j] = *reinterpret_cast<const v4i *>(src[j] + (size_t)(kt + DEPTH) * BKB);
        }
        __builtin_amdgcn_sched_barrier(0);
        __syncthreads();
#pragma unroll
        for (int ks = 0; ks < 4; ks++) {
            const v4i fa = *reinterpret_cast<const v4i *>(buf + offa + (((2 * ks + g) ^ sa) << 4));
            const v4i fw = *reinterpret_cast<const v4i *>(buf + offw + (((2 * ks + g) ^ sw) << 4));
            acc = T::mma(fw, fa, acc);
        }
    };
    int kt = 0;
    for (; kt + DEPTH < KT; kt += DEPTH)
#pragma unroll
        for (int d = 0; d < DEPTH; d++) stage(kt + d, d, true);
#pragma unroll
    for (int d = 0; d < DEPTH; d++) stage(kt + d, d, false);
    const typename Epi::Tab tb = epi.load_tab(tab, BN, wn, g);     // arrives while the waves gather
    __syncthreads();                                              // both buffers are idle from here on

    constexpr int OB = Epi::OUT_BYTES;
    constexpr int STRIDE = BN * OB + 16;
    static_assert(BM * STRIDE <= 2 * STAGE_BYTES, "staging tile does not fit");
    {
        typename Epi::pack_t pk[4];
        epi.tile(acc, tb, tab, BN, wn, g, pk);
#pragma unroll
        for (int q = 0; q < 4; q++)
            *reinterpret_cast<typename Epi::pack_t *>(lds + (wm + r) * STRIDE + (wn + 8 * q + 4 * g) * OB) = pk[q];
    }
    __syncthreads();
    constexpr int CHUNKS = BN * OB / 16;
    for (int idx = tid; idx < BM * CHUNKS; idx += NT) {
        const int lrow = idx / CHUNKS, ochunk = idx % CHUNKS;
        if (m0 + lrow < M)
            *reinterpret_cast<v4i *>(out + ((size_t)(m0 + lrow) * N + n0) * OB + ochunk * 16) =
                *reinterpret_cast<const v4i *>(lds + lrow * STRIDE + ochunk * 16);
    }
}

template <class T, class Epi, int WGN, int DEPTH>
hipError_t launch_longk(const void *A, const void *W, void *out, const Epi &epi, Rows rows, int N, int K, hipStream_t st,
                        const Timing *tm)
{
    constexpr int BN = 32 * WGN;
    const int kbytes = K * T::ELEM;
    if (N % BN || kbytes % (128 * DEPTH)) return hipErrorInvalidValue;
    const size_t LDS = 2 * (size_t)(64 + BN) * 128 + (size_t)Epi::NTAB * BN * sizeof(float);
    const int tiles_n = N / BN, tiles_m = (rows.host_rows + 63) / 64;
    launch_kernel(gemm_nt_longk_kernel<T, Epi, WGN, DEPTH>, dim3(tiles_n * tiles_m), dim3(128 * WGN), LDS, st, tm,
                  (const char *)A, (const char *)W, (char *)out, epi, rows.host_rows, rows.dev_rows, N, kbytes, tiles_n);
    return hipGetLastError();
}

// Tile configuration per problem shape.  What bounds the main loop on this chip is the rate at which
// a CU pulls operand stages out of L2 (20 to 40 bytes per clock per CU, whichever way they are loaded),
// so small problems want many small tiles (more CUs pulling), large ones the larger tile (less traffic):
//   0: 128 x 128 tile, 64-byte stages, 4-deep ring  (any K that is a multiple of 64 bytes)
//   1: 128 x 128 tile, 128-byte stages (whole cache lines per row), 2-deep ring, 2 blocks per CU
//   2: 64 tokens x 128 channels, otherwise as 1: up to about two and a half 128 x 128 tiles per CU; rows of
//      3072 bytes or more (FFN2) get a 3-deep ring (72 KB, still two blocks per CU) when there is at most one
//      block per CU: -4 % on the BERT-base forward (with more blocks than CUs it measured slower); a 4-deep ring is faster for the kernel alone but crowds out the other group's kernels
constexpr int LONG_K_BYTES = 3072;
constexpr int BIG_TILE_MIN_ROWS = 16384;                         // from here on the 256 x 256 tiles fill the chip several times over

constexpr int big_tile_width(int cfg) { return cfg == 6 ? 192 : 256; }

template <class T, class Epi>
hipError_t launch(const void *A, const void *W, void *out, const Epi &epi, Rows rows, int N, int K, hipStream_t st,
                  const Timing *tm)
{
    int cfg = gemm_config_override.load(std::memory_order_relaxed);
    const bool forced = cfg >= 0;
    const int kbytes = K * T::ELEM;
    if (cfg >= 3 && (N % big_tile_width(cfg) || kbytes % 128)) cfg = -1;   // whole columns of tiles, whole 128-byte stages
    if (cfg >= 0 && cfg < 3 && kbytes % 128) cfg = 0;
    if (cfg < 0) {
        if (kbytes % 128) cfg = 0;
        else {
            const long tiles = (long)(N / 128) * ((rows.host_rows + 127) / 128);
            // fewer 128 x 128 tiles than CUs: the smaller tiles of configuration 2 (BERT-large's 1024-wide GEMMs at
            // 4096 tokens, 256 tiles, measured -4.4 % on that forward with 128 x 128 against 64 x 128)
            cfg = tiles < 256 ? 2 : 1;
            // wide GEMMs (QKV, FFN1) from about a thousand tokens: 128 x 192 tiles, 64 x 96 per wave, two blocks
            // per CU.  Measured in the BERT-base forward at 2 x 2048 tokens: -5 % with FFN1 (whose table-lookup epilogue
            // in the 64 x 128 configuration costs more than it saves: its table in LDS takes the third resident block
            // away), another -1.4 % with QKV; the FP16 forward gains 2 %
            if (N % 192 == 0 && N >= 2304 && rows.host_rows >= 1024) cfg = 6;
            // widths that 192 does not divide (FFN1 of BERT-large, 4096): 128 x 256 tiles (-3.5 % on that forward
            // at 2 x 4096 tokens against 128 x 128; 256 x 128 -0.5 %, 64 x 128 +5.5 %)
            else if (N % 256 == 0 && N >= 2304 && rows.host_rows >= 1024) cfg = 4;
            // many tokens (INT8): wave tiles of 64 x 128 halve the LDS operand traffic per MFMA, two such blocks
            // per CU overlap one's epilogue with the other's main loop; long operand rows amortise the epilogue of a
            // 256 x 256 tile by themselves
            if (std::is_same<T, I8>::value && N % 256 == 0 && rows.host_rows >= BIG_TILE_MIN_ROWS)
                cfg = kbytes >= LONG_K_BYTES ? 7 : 4;
        }
    }
    switch (cfg) {
    case 3: return launch_big<T, Epi, 4, 4, 128, 2>(A, W, out, epi, rows, N, K, st, tm);      // 256 x 256, two 128-byte stages
    case 4: return launch_big<T, Epi, 2, 4, 64, 3, 2>(A, W, out, epi, rows, N, K, st, tm);    // 128 tokens x 256 channels, two blocks per CU
    case 5: return launch_big<T, Epi, 4, 2, 64, 3, 2>(A, W, out, epi, rows, N, K, st, tm);    // 256 tokens x 128 channels, two blocks per CU
    case 6: return launch_big<T, Epi, 2, 3, 64, 3, 2>(A, W, out, epi, rows, N, K, st, tm);    // 128 x 192, two blocks per CU
    case 7: return launch_big<T, Epi, 4, 4, 64, 4>(A, W, out, epi, rows, N, K, st, tm);       // 256 x 256, four 64-byte stages
    case 1:
        // the GELU epilogue is as much vector work as the main loop is matrix work: 64-byte stages leave room
        // for three resident blocks per CU, whose epilogues and main loops overlap (-3 % on the large forwards)
        if constexpr (std::is_same<Epi, EpiGeluQuant>::value || std::is_same<Epi, EpiGeluTable>::value)
            return launch_cfg<T, Epi, 2, 2, 64, 3, 3>(A, W, out, epi, rows, N, K, st, tm);
        else return launch_cfg<T, Epi, 2, 2, 128, 2, 2>(A, W, out, epi, rows, N, K, st, tm);
    case 2: {
        const long row_tiles = (rows.host_rows + 63) / 64;
        const bool long_k = K * T::ELEM >= LONG_K_BYTES;
        // 64 x 96 tiles (six waves of 32 x 32) when they put the problem on more CUs without exceeding one block
        // per CU: the rate at which one CU pulls operands is what bounds these small problems
        if (!forced && N % 96 == 0 && (N / 96) * row_tiles <= 256) {
            // (measured in the BERT-base forward at 2 x 2048 tokens: two stages held in registers -2 %, three +11 %,
            // six +3 % against the three-deep LDS ring, although six is the fastest alone: 12.3 against 14.2 us)
            if constexpr (Epi::STAGED && !std::is_same<Epi, EpiGeluTable>::value) {
                // (also for short rows: the attention-output GEMM; same speed in the batch-32 forward, -4 % for one sequence)
                if (kbytes % 256 == 0) return launch_longk<T, Epi, 3, 2>(A, W, out, epi, rows, N, K, st, tm);
            }
            if (long_k) return launch_cfg<T, Epi, 1, 1, 128, 3, 2, 2, 3>(A, W, out, epi, rows, N, K, st, tm);
            return launch_cfg<T, Epi, 1, 1, 128, 2, 2, 2, 3>(A, W, out, epi, rows, N, K, st, tm);
        }
        if constexpr (Epi::STAGED && !std::is_same<Epi, EpiGeluTable>::value) {
            if (!forced && long_k && kbytes % 256 == 0 && (N / 128) * row_tiles <= 256)
                return launch_longk<T, Epi, 4, 2>(A, W, out, epi, rows, N, K, st, tm);
        }
        if (long_k && (N / 128) * row_tiles <= 256) return launch_cfg<T, Epi, 1, 2, 128, 3, 2>(A, W, out, epi, rows, N, K, st, tm);
        return launch_cfg<T, Epi, 1, 2, 128, 2, 2>(A, W, out, epi, rows, N, K, st, tm);
    }
    default: return launch_cfg<T, Epi, 2, 2, 64, 4, 2>(A, W, out, epi, rows, N, K, st, tm);
    }
}

}  // namespace

std::atomic<int> gemm_config_override{-1};                    // tuning aid: force one tile configuration (see launch())

hipError_t launch_gemm_i8(GemmEpilogue epi, const int8_t *A, const int8_t *W, void *out, const float *m, const float *b,
                          float inv_s_out, const GeluTable *gt, Rows rows, int N, int K, hipStream_t st, const Timing *tm)
{
    switch (epi) {
    case EPI_RAW_I32: return launch<I8>(A, W, out, EpiRawI32{(int32_t *)out, N}, rows, N, K, st, tm);
    case EPI_REQUANT: return launch<I8>(A, W, out, EpiRequant{m, b}, rows, N, K, st, tm);
    case EPI_GELU_QUANT:
        if (gt && gt->entries)
            return launch<I8>(A, W, out, EpiGeluTable{m, b, gt->entries, gt->spec.rate, gt->spec.offset, gt->spec.t_max, gt->spec.bins},
                              rows, N, K, st, tm);
        return launch<I8>(A, W, out, EpiGeluQuant{m, b, inv_s_out}, rows, N, K, st, tm);
    }
    return hipErrorInvalidValue;
}

hipError_t launch_gemm_f16(const __half *A, const __half *W, const float *bias, bool gelu, __half *out, Rows rows,
                           int N, int K, hipStream_t st, const Timing *tm)
{
    return launch<F16>(A, W, out, EpiF16{bias, gelu}, rows, N, K, st, tm);
}

}  // namespace samp
