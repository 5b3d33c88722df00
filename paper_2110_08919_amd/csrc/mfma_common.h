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

// s_waitcnt vmcnt(n) with n a run-time value in 0..15 (other counters untouched).
__device__ __forceinline__ void wait_vmcnt(int n)
{
    switch (n) {
    case 0: __builtin_amdgcn_s_waitcnt(0x0F70); break;
    case 1: __builtin_amdgcn_s_waitcnt(0x0F71); break;
    case 2: __builtin_amdgcn_s_waitcnt(0x0F72); break;
    case 3: __builtin_amdgcn_s_waitcnt(0x0F73); break;
    case 4: __builtin_amdgcn_s_waitcnt(0x0F74); break;
    case 5: __builtin_amdgcn_s_waitcnt(0x0F75); break;
    case 6: __builtin_amdgcn_s_waitcnt(0x0F76); break;
    case 7: __builtin_amdgcn_s_waitcnt(0x0F77); break;
    case 8: __builtin_amdgcn_s_waitcnt(0x0F78); break;
    case 9: __builtin_amdgcn_s_waitcnt(0x0F79); break;
    case 10: __builtin_amdgcn_s_waitcnt(0x0F7A); break;
    case 11: __builtin_amdgcn_s_waitcnt(0x0F7B); break;
    case 12: __builtin_amdgcn_s_waitcnt(0x0F7C); break;
    case 13: __builtin_amdgcn_s_waitcnt(0x0F7D); break;
    case 14: __builtin_amdgcn_s_waitcnt(0x0F7E); break;
    default: __builtin_amdgcn_s_waitcnt(0x0F7F); break;
    }
}

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
