// Wave-wide minimum / maximum in every lane.  The first four butterfly steps (partners inside a
// row of 16 lanes) go through data-parallel-primitive moves, which take a few cycles; only the two
// steps across rows pay the LDS round trip of a lane permute.  All 64 lanes must be active.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lpq {

// DPP controls: quad_perm [1,0,3,2] and [2,3,0,1] (partner lane ^ 1, lane ^ 2), mirror inside
// half a row (quad 0 <-> quad 1 of each 8 lanes), mirror inside a row (the two halves of 16 lanes).
constexpr int DPP_XOR1 = 0xB1, DPP_XOR2 = 0x4E, DPP_HALF_MIRROR = 0x141, DPP_ROW_MIRROR = 0x140;

template <int CTRL>
__device__ __forceinline__ int dpp_move(int v)
{
    return __builtin_amdgcn_update_dpp(v, v, CTRL, 0xF, 0xF, false);
}

template <int CTRL>
__device__ __forceinline__ uint64_t dpp_move64(uint64_t v)
{
    const int lo = dpp_move<CTRL>((int)(uint32_t)v), hi = dpp_move<CTRL>((int)(uint32_t)(v >> 32));
    return ((uint64_t)(uint32_t)hi << 32) | (uint32_t)lo;
}

__device__ __forceinline__ uint64_t wave_min_u64(uint64_t c)
{
    uint64_t t;
    t = dpp_move64<DPP_XOR1>(c);        c = t < c ? t : c;
    t = dpp_move64<DPP_XOR2>(c);        c = t < c ? t : c;
    t = dpp_move64<DPP_HALF_MIRROR>(c); c = t < c ? t : c;
    t = dpp_move64<DPP_ROW_MIRROR>(c);  c = t < c ? t : c;
    t = __shfl_xor(c, 16, 64);          c = t < c ? t : c;
    t = __shfl_xor(c, 32, 64);          c = t < c ? t : c;
    return c;
}

__device__ __forceinline__ int wave_max_i32(int v)
{
    int t;
    t = dpp_move<DPP_XOR1>(v);        v = t > v ? t : v;
    t = dpp_move<DPP_XOR2>(v);        v = t > v ? t : v;
    t = dpp_move<DPP_HALF_MIRROR>(v); v = t > v ? t : v;
    t = dpp_move<DPP_ROW_MIRROR>(v);  v = t > v ? t : v;
    t = __shfl_xor(v, 16, 64);        v = t > v ? t : v;
    t = __shfl_xor(v, 32, 64);        v = t > v ? t : v;
    return v;
}

__device__ __forceinline__ int wave_min_i32(int v) { return -wave_max_i32(-v); }

}  // namespace lpq
