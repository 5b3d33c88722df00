// Kernels that work on candidate lists instead of the whole corpus.
//
// gather_dist_kernel: the integer distance phi(Q(q), Q(x_id)) between a query and the items an
// id list names - the distance routine Section 5.2 swaps into graph indexes - as a batched
// gather: 8 lanes fetch one 16-byte-chunked code row, v_dot4 products, the squared distance
// through the exact integer identity |cq|^2 + |cx|^2 - 2 cq.cx with the stored item norms.
//
// rerank_f32_kernel: second stage that recovers the recall lost to quantization (the 2-6 % of
// Section 5.3): exact distances of each query's kc candidates on the original fp32 vectors,
// accumulated in binary64, sorted by (distance, id), the k best written out.
#include "lpq_internal.h"

namespace lpq {

namespace {

constexpr int GD_THREADS = 256;
constexpr int GD_ITEMS = 256;   // items of one query per workgroup (8 passes of 32)

__global__ __launch_bounds__(GD_THREADS) void gather_dist_kernel(
    const int8_t *__restrict__ codes, const int32_t *__restrict__ norms, int64_t n, int d, int d_pad,
    const int8_t *__restrict__ q, int64_t ldq, const int32_t *__restrict__ ids, int m, int blocks_per_query,
    int metric, int32_t *__restrict__ out, bool packed)
{
    extern __shared__ __align__(16) unsigned char smem[];
    uint4 *qs = reinterpret_cast<uint4 *>(smem);   // the query's codes, zero padded to d_pad
    const int64_t qi = blockIdx.x / blocks_per_query;
    const int j0 = (blockIdx.x % blocks_per_query) * GD_ITEMS;
    int8_t *qb = reinterpret_cast<int8_t *>(smem);
    // Packed rows (two codes per byte, stored + 8): the query saturates to -8 .. 7 like the items,
    // and each group of 8 of its codes is stored evens first (0 2 4 6 1 3 5 7), so that the low
    // nibbles of a packed dword meet one query dword and its high nibbles the next.
    for (int c = threadIdx.x; c < d_pad; c += GD_THREADS) {
        int v = (c < d) ? (int)q[qi * ldq + c] : 0;
        int at = c;
        if (packed) {
            v = v < -8 ? -8 : (v > 7 ? 7 : v);
            at = (c & ~7) + ((c & 1) ? 4 : 0) + ((c & 7) >> 1);
        }
        qb[at] = (int8_t)v;
    }
    __syncthreads();
    const int sub = threadIdx.x & 7, grp = threadIdx.x >> 3;
    const int chunks = d_pad >> 4;
    const bool l2 = metric == LPQ_METRIC_L2SQ;
    for (int p = 0; p < GD_ITEMS / 32; ++p) {
        const int j = j0 + p * 32 + grp;
        const int32_t id = (j < m) ? ids[qi * m + j] : -1;
        const bool live = id >= 0 && (int64_t)id < n;
        int dot = 0, qq = 0;
        if (live && packed) {
            const uint4 *xr = reinterpret_cast<const uint4 *>(codes + (int64_t)id * (d_pad >> 1));
            const unsigned mk = 0x0F0F0F0Fu;
            int sq = 0;
            for (int c = sub; c < (chunks >> 1); c += 8) {
                const uint4 xv = xr[c], q0 = qs[2 * c], q1 = qs[2 * c + 1];
                dot = __builtin_amdgcn_sdot4((int)(xv.x & mk), (int)q0.x, dot, false);
                dot = __builtin_amdgcn_sdot4((int)((xv.x >> 4) & mk), (int)q0.y, dot, false);
                dot = __builtin_amdgcn_sdot4((int)(xv.y & mk), (int)q0.z, dot, false);
                dot = __builtin_amdgcn_sdot4((int)((xv.y >> 4) & mk), (int)q0.w, dot, false);
                dot = __builtin_amdgcn_sdot4((int)(xv.z & mk), (int)q1.x, dot, false);
                dot = __builtin_amdgcn_sdot4((int)((xv.z >> 4) & mk), (int)q1.y, dot, false);
                dot = __builtin_amdgcn_sdot4((int)(xv.w & mk), (int)q1.z, dot, false);
                dot = __builtin_amdgcn_sdot4((int)((xv.w >> 4) & mk), (int)q1.w, dot, false);
                const unsigned qv[8] = {q0.x, q0.y, q0.z, q0.w, q1.x, q1.y, q1.z, q1.w};
#pragma unroll
                for (int t = 0; t < 8; ++t) {
                    qq = __builtin_amdgcn_sdot4((int)qv[t], (int)qv[t], qq, false);
                    sq = __builtin_amdgcn_sdot4((int)qv[t], 0x01010101, sq, false);
                }
            }
            dot -= 8 * sq;   // the stored nibbles are code + 8
        } else if (live) {
            const uint4 *xr = reinterpret_cast<const uint4 *>(codes + (int64_t)id * d_pad);
            for (int c = sub; c < chunks; c += 8) {
                const uint4 xv = xr[c], qv = qs[c];
                dot = __builtin_amdgcn_sdot4((int)xv.x, (int)qv.x, dot, false);
                dot = __builtin_amdgcn_sdot4((int)xv.y, (int)qv.y, dot, false);
                dot = __builtin_amdgcn_sdot4((int)xv.z, (int)qv.z, dot, false);
                dot = __builtin_amdgcn_sdot4((int)xv.w, (int)qv.w, dot, false);
                qq = __builtin_amdgcn_sdot4((int)qv.x, (int)qv.x, qq, false);
                qq = __builtin_amdgcn_sdot4((int)qv.y, (int)qv.y, qq, false);
                qq = __builtin_amdgcn_sdot4((int)qv.z, (int)qv.z, qq, false);
                qq = __builtin_amdgcn_sdot4((int)qv.w, (int)qv.w, qq, false);
            }
        }
        dot += __shfl_xor(dot, 4, 64); qq += __shfl_xor(qq, 4, 64);
        dot += __shfl_xor(dot, 2, 64); qq += __shfl_xor(qq, 2, 64);
        dot += __shfl_xor(dot, 1, 64); qq += __shfl_xor(qq, 1, 64);
        if (sub == 0 && j < m) {
            int32_t v;
            if (!live) v = l2 ? INT32_MAX : INT32_MIN;
            else v = l2 ? qq + norms[id] - 2 * dot : dot;
            out[qi * m + j] = v;
        }
    }
}

// ---------------------------------------------------------------------- re-rank ----
constexpr int RR_THREADS = 256;

__device__ __forceinline__ unsigned long long double_to_sortable(double v)
{
    unsigned long long u = (unsigned long long)__double_as_longlong(v);
    return (u >> 63) ? ~u : (u | 0x8000000000000000ull);
}
__device__ __forceinline__ double sortable_to_double(unsigned long long u)
{
    u = (u >> 63) ? (u & 0x7fffffffffffffffull) : ~u;
    return __longlong_as_double((long long)u);
}

__global__ __launch_bounds__(RR_THREADS) void rerank_f32_kernel(
    const float *__restrict__ x, int64_t n, int64_t ldx, const float *__restrict__ q, int64_t ldq, int d,
    const int32_t *__restrict__ cand, int kc, int cap, int k, int metric, int32_t *__restrict__ ids,
    float *__restrict__ dists)
{
    extern __shared__ __align__(16) unsigned char smem[];
    unsigned long long *key = reinterpret_cast<unsigned long long *>(smem);   // [cap]
    int32_t *idv = reinterpret_cast<int32_t *>(key + cap);                    // [cap]
    const int64_t qi = blockIdx.x;
    const float *qr = q + qi * ldq;
    const bool l2 = metric == LPQ_METRIC_L2SQ;
    const int sub = threadIdx.x & 7, grp = threadIdx.x >> 3;
    for (int j0 = 0; j0 < cap; j0 += RR_THREADS / 8) {
        const int j = j0 + grp;
        const int32_t id = (j < kc) ? cand[qi * kc + j] : -1;
        const bool live = id >= 0 && (int64_t)id < n;
        double s = 0.0;
        if (live) {
            const float *xr = x + (int64_t)id * ldx;
            for (int t = sub; t < d; t += 8) {
                const double a = (double)qr[t], b = (double)xr[t];
                if (l2) { const double df = a - b; s += df * df; }
                else s += a * b;
            }
        }
        s += __shfl_xor(s, 4, 64);
        s += __shfl_xor(s, 2, 64);
        s += __shfl_xor(s, 1, 64);
        if (sub == 0 && j < cap) {
            key[j] = live ? double_to_sortable(l2 ? s : -s) : ~0ull;
            idv[j] = live ? id : INT32_MAX;   // absent entries sort last
        }
    }
    __syncthreads();
    // ascending bitonic sort of (key, id) pairs
    for (int size = 2; size <= cap; size <<= 1)
        for (int stride = size >> 1; stride > 0; stride >>= 1) {
            for (int i = threadIdx.x; i < (cap >> 1); i += RR_THREADS) {
                const int lo = 2 * i - (i & (stride - 1)), hi = lo + stride;
                const bool up = (lo & size) == 0;
                const unsigned long long ka = key[lo], kb = key[hi];
                const int32_t ia = idv[lo], ib = idv[hi];
                const bool gt = ka > kb || (ka == kb && ia > ib);
                if (gt == up) { key[lo] = kb; key[hi] = ka; idv[lo] = ib; idv[hi] = ia; }
            }
            __syncthreads();
        }
    for (int r = threadIdx.x; r < k; r += RR_THREADS) {
        const bool have = r < cap && key[r] != ~0ull;
        ids[qi * k + r] = have ? idv[r] : -1;
        float v = l2 ? INFINITY : -INFINITY;
        if (have) { const double s = sortable_to_double(key[r]); v = (float)(l2 ? s : -s); }
        dists[qi * k + r] = v;
    }
}

}  // namespace

hipError_t launch_gather_dist(const int8_t *codes, const int32_t *norms, int64_t n, int d, int d_pad, const int8_t *q,
                              int64_t nq, int64_t ldq, const int32_t *ids, int m, int metric, int32_t *out,
                              hipStream_t st, bool packed)
{
    if (nq <= 0 || m <= 0) return hipSuccess;
    const int bpq = (int)ceil_div(m, GD_ITEMS);
    if (nq * bpq >= (int64_t(1) << 31)) return hipErrorInvalidValue;
    gather_dist_kernel<<<(unsigned)(nq * bpq), GD_THREADS, (size_t)d_pad, st>>>(codes, norms, n, d, d_pad, q, ldq, ids, m,
                                                                               bpq, metric, out, packed);
    return hipGetLastError();
}

hipError_t launch_rerank_f32(const float *x, int64_t n, int64_t ldx, const float *q, int64_t nq, int64_t ldq, int d,
                             const int32_t *cand, int kc, int k, int metric, int32_t *ids, float *dists, hipStream_t st)
{
    if (nq <= 0) return hipSuccess;
    const int cap = next_pow2(kc < 32 ? 32 : kc);   // a whole number of 32-candidate passes
    if (cap > 4096) return hipErrorInvalidValue;
    rerank_f32_kernel<<<(unsigned)nq, RR_THREADS, (size_t)cap * 12, st>>>(x, n, ldx, q, ldq, d, cand, kc, cap, k, metric,
                                                                         ids, dists);
    return hipGetLastError();
}

}  // namespace lpq
