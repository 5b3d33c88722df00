// Workgroup-level selection helpers shared by the scan kernels and the merge kernel.
#pragma once

#include "lpq_internal.h"

namespace lpq {

// Ascending bitonic sort of buf[0..cap) (cap a power of two) by all threads of the block.
__device__ inline void block_bitonic_sort(cand_t *buf, int cap)
{
    for (int size = 2; size <= cap; size <<= 1) {
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int i = threadIdx.x; i < (cap >> 1); i += blockDim.x) {
                const int lo = 2 * i - (i & (stride - 1));
                const int hi = lo + stride;
                const bool up = (lo & size) == 0;
                const cand_t a = buf[lo], b = buf[hi];
                if ((a > b) == up) { buf[lo] = b; buf[hi] = a; }
            }
            __syncthreads();
        }
    }
}

// Compacts a candidate buffer that may overflow on the next step: sort, keep the best k,
// tighten the threshold to the k-th best.  Must be reached by all threads of the block;
// `need` is the largest number of appends one step can make.
__device__ inline void block_compact_if_full(cand_t *buf, int cap, int k, int need, int *s_count, cand_t *s_thr)
{
    if (*s_count + need > cap) {  // uniform: the count is stable after the caller's barrier
        block_bitonic_sort(buf, cap);
        const int cnt = *s_count < k ? *s_count : k;
        for (int i = cnt + threadIdx.x; i < cap; i += blockDim.x) buf[i] = CAND_NONE;
        if (threadIdx.x == 0) {
            if (cnt == k && buf[k - 1] < *s_thr) *s_thr = buf[k - 1];
            *s_count = cnt;
        }
        __syncthreads();
    }
}

}  // namespace lpq
