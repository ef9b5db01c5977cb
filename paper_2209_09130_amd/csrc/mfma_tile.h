// Pieces of the LDS-staged MFMA tile loop that more than one kernel file uses: the chunk swizzle of a stage row,
// explicit waits, and operand-fragment reads with waits of their own.
#pragma once
#include "samp_common.h"

#include <utility>

namespace samp {
namespace {

// XOR swizzle of the 16-byte chunk index inside an LDS row of BKB bytes (BKB = 64: 4 chunks,
// BKB = 128: 8 chunks), chosen so that the lanes of one ds_read_b128 phase hit distinct banks.
template <int BKB>
__device__ __forceinline__ int swz(int row)
{
    if constexpr (BKB == 64) return ((row >> 1) & 3) ^ ((row >> 3) & 1);
    else return (row & 7) ^ ((row >> 3) & 1);
}

// wait until at most N vector-memory operations of this wave are outstanding and all of its LDS
// reads have returned, then barrier.  The "memory" clobber keeps the compiler from moving LDS
// accesses across it.
template <int N>
__device__ __forceinline__ void wait_vm_and_barrier()
{
    static_assert(N >= 0 && N < 64, "vmcnt range");
    asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(N) : "memory");
}

// Fragment fetches of the large-tile kernel are written as ds_read_b128 instructions of its own, with
// explicit waits: left to the compiler, every group of MFMAs is preceded by a wait for ALL outstanding
// LDS reads, including the ones just issued for the step after it, which puts the LDS latency in front
// of every step instead of behind the MFMAs of the step before.  tie() makes later uses of a fragment
// depend on the wait that precedes it (an empty instruction that "rewrites" the register).
template <int OFFSET> __device__ __forceinline__ v4i lds_read128(unsigned addr)
{
    v4i v;
    asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(v) : "v"(addr), "n"(OFFSET));
    return v;
}
template <int STRIDE, int N, int... I>
__device__ __forceinline__ void lds_read_frags(unsigned addr, v4i (&f)[N], std::integer_sequence<int, I...>)
{
    ((f[I] = lds_read128<I * STRIDE>(addr)), ...);
}
__device__ __forceinline__ int tie_one(v4i &f)
{
    asm volatile("" : "+v"(f));
    return 0;
}
template <int N, int... I> __device__ __forceinline__ void tie(v4i (&f)[N], std::integer_sequence<int, I...>)
{
    (void)(tie_one(f[I]) + ... + 0);
}
template <int N> __device__ __forceinline__ void wait_lds_reads()
{
    static_assert(N >= 0 && N < 16, "lgkmcnt range");
    asm volatile("s_waitcnt lgkmcnt(%0)" ::"n"(N) : "memory");
}

}  // namespace
}  // namespace samp
