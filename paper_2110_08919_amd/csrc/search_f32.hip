// Exact search on the original fp32 vectors: the reference set S_E of the recall definition
// (Section 5.3).  The squared distance is summed directly as (q - x)^2 in fp32 (fused
// multiply-add, partial sums per lane combined by a tree), never through the norm identity,
// so near neighbours keep their relative accuracy.  One workgroup per (query, corpus split);
// selection and merge are the ones of the integer path, on an order-preserving integer image
// of the float.
#include "block_select.h"
#include "lpq_internal.h"

namespace lpq {

namespace {

constexpr int F32_THREADS = 256;
constexpr int F32_ROWS = F32_THREADS / 8;  // 8 lanes share a row, 4 floats each per step

template <bool VEC>
__global__ __launch_bounds__(F32_THREADS) void search_f32_kernel(
    const float *__restrict__ x, int64_t n, int64_t ldx, const float *__restrict__ qv, int64_t ldq, int d,
    int k, int mode, int S, int64_t split_rows, cand_t *__restrict__ lists, int cap)
{
    extern __shared__ __align__(16) unsigned char smem[];
    cand_t *buf = reinterpret_cast<cand_t *>(smem);
    float *qs = reinterpret_cast<float *>(buf + cap);
    __shared__ int s_count;
    __shared__ cand_t s_thr;

    const int64_t q = blockIdx.x / S;
    const int s = blockIdx.x % S;
    const int chunks = (d + 3) >> 2;
    const int64_t rs = (int64_t)s * split_rows;
    const int64_t re = (rs + split_rows < n) ? rs + split_rows : n;
    const bool l2 = mode == MODE_F32_L2;

    for (int c = threadIdx.x; c < 4 * chunks; c += F32_THREADS) qs[c] = (c < d) ? qv[q * ldq + c] : 0.0f;
    for (int i = threadIdx.x; i < cap; i += F32_THREADS) buf[i] = CAND_NONE;
    if (threadIdx.x == 0) { s_count = 0; s_thr = CAND_NONE; }
    __syncthreads();

    const int sub = threadIdx.x & 7, grp = threadIdx.x >> 3;
    for (int64_t base = rs; base < re; base += F32_ROWS) {
        const int64_t row = base + grp;
        float acc = 0.0f;
        if (row < re) {
            const float *xr = x + row * ldx;
            for (int c = sub; c < chunks; c += 8) {
                float xv[4];
                if (VEC && 4 * c + 3 < d) {
                    const float4 t = *reinterpret_cast<const float4 *>(xr + 4 * c);
                    xv[0] = t.x; xv[1] = t.y; xv[2] = t.z; xv[3] = t.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) xv[j] = (4 * c + j < d) ? xr[4 * c + j] : 0.0f;
                }
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const float qq = qs[4 * c + j];
                    if (l2) { const float t = qq - xv[j]; acc = fmaf(t, t, acc); }
                    else acc = fmaf(qq, xv[j], acc);
                }
            }
        }
        acc += __shfl_xor(acc, 4, 64);
        acc += __shfl_xor(acc, 2, 64);
        acc += __shfl_xor(acc, 1, 64);
        if (sub == 0 && row < re) {
            const cand_t c = make_cand(float_to_sortable(l2 ? acc : -acc), (uint32_t)row);
            if (c < s_thr) {
                const int pos = atomicAdd(&s_count, 1);
                buf[pos] = c;
            }
        }
        __syncthreads();
        block_compact_if_full(buf, cap, k, F32_ROWS, &s_count, &s_thr);
    }
    block_bitonic_sort(buf, cap);
    cand_t *out = lists + ((int64_t)q * S + s) * k;
    for (int i = threadIdx.x; i < k; i += F32_THREADS) out[i] = buf[i];
}

int f32_splits(int64_t n, int64_t nq, int k)
{
    int64_t s = ceil_div(2048, nq > 0 ? nq : 1);
    const int64_t by_rows = n / 2048 > 0 ? n / 2048 : 1;
    if (s > by_rows) s = by_rows;
    if (s > merge_max_lists(k)) s = merge_max_lists(k);
    return (int)(s < 1 ? 1 : s);
}

}  // namespace

size_t f32_workspace_bytes(int64_t n, int64_t nq, int d, int k)
{
    (void)d;
    return (size_t)nq * f32_splits(n, nq, k) * k * sizeof(cand_t);
}

hipError_t launch_search_f32(const float *x, int64_t n, int64_t ldx, const float *q, int64_t nq, int64_t ldq,
                             int d, int k, int metric, int32_t *ids, float *dists, void *ws, hipStream_t st)
{
    const int S = f32_splits(n, nq, k);
    const int mode = metric == LPQ_METRIC_L2SQ ? MODE_F32_L2 : MODE_F32_IP;
    const int cap = next_pow2((2 * k > k + 2 * F32_ROWS) ? 2 * k : k + 2 * F32_ROWS);
    const int64_t split_rows = round_up(ceil_div(n, S), F32_ROWS);
    const size_t shmem = (size_t)cap * sizeof(cand_t) + (size_t)((d + 3) / 4) * 16;
    if (shmem > 64 * 1024) return hipErrorInvalidValue;
    cand_t *lists = reinterpret_cast<cand_t *>(ws);
    const bool vec = ((uintptr_t)x % 16 == 0) && (ldx % 4 == 0);
    if (vec)
        search_f32_kernel<true><<<(unsigned)(nq * S), F32_THREADS, shmem, st>>>(x, n, ldx, q, ldq, d, k, mode, S,
                                                                                 split_rows, lists, cap);
    else
        search_f32_kernel<false><<<(unsigned)(nq * S), F32_THREADS, shmem, st>>>(x, n, ldx, q, ldq, d, k, mode, S,
                                                                                  split_rows, lists, cap);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    return launch_merge(lists, nq, S, k, nullptr, nullptr, nullptr, ids, reinterpret_cast<int32_t *>(dists),
                        nullptr, mode, st, true);
}

}  // namespace lpq
