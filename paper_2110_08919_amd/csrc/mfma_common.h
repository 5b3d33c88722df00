// Pieces shared by the two matrix-core search kernels (gfx950 only).
#pragma once

#include "lpq_internal.h"

namespace lpq {

namespace {

typedef int v2i __attribute__((ext_vector_type(2)));
typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int WAVES = 4;
constexpr int THREADS = WAVES * 64;
constexpr int NSTG = 4;    // LDS ring depth
constexpr int QCAP = 64;   // dumps a wave can queue; one epilogue makes at most 64

// Orders the LDS traffic of the lanes of one wave (a wave's LDS instructions execute in
// issue order, so this only has to stop the compiler from moving accesses across it).  It does
// not touch the vector-memory counter: asynchronous stage copies stay in flight.
__device__ __forceinline__ void wave_lds_sync()
{
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_wave_barrier();
}

// Asynchronous 16-byte-per-lane copy global -> LDS: lane l of the wave writes LDS bytes
// [base + 16 l, base + 16 l + 16).  `base` must be wave-uniform.  The copy is tracked by the
// vector-memory counter only; the caller orders it with wait_vmcnt() and a barrier.
__device__ __forceinline__ void async_copy16(const void *gptr, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}
__device__ __forceinline__ void async_copy4(const void *gptr, unsigned lds_base)
{
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, off" ::"s"(lds_base), "v"(gptr) : "memory");
}
__device__ __forceinline__ unsigned lds_offset(const void *p)
{
    return (unsigned)(uintptr_t)(__attribute__((address_space(3))) const void *)p;
}

// s_waitcnt vmcnt(n) with n a run-time value in 0..63 (other counters untouched).  The count is
// an immediate, split over bits 3:0 and 15:14 of the operand.
constexpr int vmcnt_imm(int n) { return 0x0F70 | (n & 15) | ((n >> 4) << 14); }   // operand of s_waitcnt vmcnt(n)
#define LPQ_WAITCNT_CASE(N) case N: __builtin_amdgcn_s_waitcnt(0x0F70 | ((N) & 15) | (((N) >> 4) << 14)); break;
#define LPQ_WAITCNT_CASES8(B) LPQ_WAITCNT_CASE(B) LPQ_WAITCNT_CASE(B + 1) LPQ_WAITCNT_CASE(B + 2) LPQ_WAITCNT_CASE(B + 3) \
    LPQ_WAITCNT_CASE(B + 4) LPQ_WAITCNT_CASE(B + 5) LPQ_WAITCNT_CASE(B + 6) LPQ_WAITCNT_CASE(B + 7)
__device__ __forceinline__ void wait_vmcnt(int n)
{
    switch (n) {
    LPQ_WAITCNT_CASES8(0) LPQ_WAITCNT_CASES8(8) LPQ_WAITCNT_CASES8(16) LPQ_WAITCNT_CASES8(24)
    LPQ_WAITCNT_CASES8(32) LPQ_WAITCNT_CASES8(40) LPQ_WAITCNT_CASES8(48)
    LPQ_WAITCNT_CASE(56) LPQ_WAITCNT_CASE(57) LPQ_WAITCNT_CASE(58) LPQ_WAITCNT_CASE(59) LPQ_WAITCNT_CASE(60)
    LPQ_WAITCNT_CASE(61) LPQ_WAITCNT_CASE(62)
    default: __builtin_amdgcn_s_waitcnt(0xCF7F); break;   // 63: the counter's maximum
    }
}
#undef LPQ_WAITCNT_CASES8
#undef LPQ_WAITCNT_CASE

// A candidate can only beat the threshold candidate c if its E is >= thr_e(c).
__device__ inline int thr_e(cand_t c)
{
    if (c == CAND_NONE) return INT32_MIN;
    if (c == 0) return INT32_MAX;  // a query slot that must never collect anything
    const long long t = (-(long long)cand_key(c)) >> 1;
    return t > INT32_MAX ? INT32_MAX : (t < INT32_MIN ? INT32_MIN : (int)t);
}

// Swizzle of the 16-byte chunk slots of LDS row i (SLOTS slots per row, a power of two):
// chunk c of row i lives in slot c ^ swz(i).  Conflict-free for ds_read_b128 of one chunk
// column by 32 consecutive rows, with 32 or 64 LDS banks.
template <int SLOTS>
__device__ __forceinline__ int swz(int i)
{
    if (SLOTS == 16) return i & 15;
    constexpr int A = SLOTS == 8 ? 0 : (SLOTS == 4 ? 1 : 2);
    return ((i >> A) ^ (i >> 3)) & (SLOTS - 1);
}

}  // namespace

}  // namespace lpq
