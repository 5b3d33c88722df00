// Exact search on the original fp32 vectors: the reference set S_E of the recall definition
// (Section 5.3).  The squared distance is summed directly as (q - x)^2 in fp32 (fused
// multiply-add, partial sums per lane combined by a tree), never through the norm identity,
// so near neighbours keep their relative accuracy.  One workgroup per (query tile, corpus split);
// selection and merge are the ones of the integer path, on an order-preserving integer image
// of the float.
#include "block_select.h"
#include "lpq_internal.h"
#include "wave_ops.h"

namespace lpq {

namespace {

constexpr int F32_THREADS = 256;
constexpr int F32_ROWS = F32_THREADS / 8;  // 8 lanes share a row, 4 floats each per step

// QT queries share one pass over the rows of a split and every lane group works on F32_R rows at
// once: the corpus is read once per QT queries, and a query value fetched from LDS feeds F32_R
// subtract/multiply-add pairs (with one row per group the LDS pipe, not the VALU, was the limit).
constexpr int F32_R = 4;
constexpr int F32_STEP = F32_ROWS * F32_R;   // rows per step of a workgroup

// One step of the halving butterfly over lane pairs: of its first CNT partial sums a lane keeps
// one half (the upper one if `upper`), adds the partner's partial sums of that half and leaves the
// results in red[0 .. CNT/2).  With a single sum left it is a plain exchange.  The partner is given
// by a DPP control (no LDS round trip): it must differ from the lane in the bit that `upper` tests
// and lie in the same group of 8 lanes; which other bits differ does not matter for the sums.
template <int CNT, int CTRL, int N>
__device__ __forceinline__ void halve_sums(float (&red)[N], bool upper)
{
    if constexpr (CNT > 1) {
        constexpr int H = CNT / 2;
#pragma unroll
        for (int i = 0; i < H; ++i) {
            const float mine = upper ? red[H + i] : red[i];
            const float theirs = upper ? red[i] : red[H + i];
            red[i] = mine + __int_as_float(dpp_move<CTRL>(__float_as_int(theirs)));
        }
    } else {
        red[0] += __int_as_float(dpp_move<CTRL>(__float_as_int(red[0])));
    }
}

// L2 is a template parameter: as a run-time flag the compiler computed both metrics for every pair
// and selected one (four vector operations per pair instead of two).
template <bool VEC, int QT, bool L2>
__global__ __launch_bounds__(F32_THREADS) void search_f32_kernel(
    const float *__restrict__ x, int64_t n, int64_t ldx, const float *__restrict__ qv, int64_t ldq, int64_t nq,
    int d, int k, int mode, int S, int64_t split_rows, cand_t *__restrict__ lists, int cap)
{
    extern __shared__ __align__(16) unsigned char smem[];
    cand_t *buf = reinterpret_cast<cand_t *>(smem);                 // [QT][cap]
    float *qs = reinterpret_cast<float *>(buf + (size_t)QT * cap);  // [QT][dp]
    __shared__ int s_count[QT];
    __shared__ cand_t s_thr[QT];

    // Workgroups are dealt round-robin to the 8 XCDs: give each XCD a contiguous range of (split,
    // query tile) pairs, split-major, so the query tiles that stream one split share that XCD's L2.
    const int tiles = gridDim.x / S, per = gridDim.x / 8, b = blockIdx.x;
    const int wk = (b < per * 8) ? (b % 8) * per + b / 8 : b;
    const int64_t q0 = (int64_t)(wk % tiles) * QT;
    const int s = wk / tiles;
    const int chunks = (d + 3) >> 2, dp = 4 * chunks;
    const int64_t rs = (int64_t)s * split_rows;
    const int64_t re = (rs + split_rows < n) ? rs + split_rows : n;
    constexpr bool l2 = L2;
    (void)mode;

    for (int i = threadIdx.x; i < QT * dp; i += F32_THREADS) {
        const int j = i / dp, c = i % dp;
        qs[i] = (c < d && q0 + j < nq) ? qv[(q0 + j) * ldq + c] : 0.0f;
    }
    for (int i = threadIdx.x; i < QT * cap; i += F32_THREADS) buf[i] = CAND_NONE;
    if (threadIdx.x < QT) { s_count[threadIdx.x] = 0; s_thr[threadIdx.x] = CAND_NONE; }
    __syncthreads();

    const int sub = threadIdx.x & 7, grp = threadIdx.x >> 3;
    for (int64_t base = rs; base < re; base += F32_STEP) {
        float acc[QT][F32_R];
#pragma unroll
        for (int j = 0; j < QT; ++j)
#pragma unroll
            for (int r = 0; r < F32_R; ++r) acc[j][r] = 0.0f;
        // Four column chunks (of 4 floats) per lane at a time: all their loads are issued before the
        // arithmetic starts, so one memory round trip covers 16 loads per lane.
        for (int cb = sub; cb < chunks; cb += 32) {
            float xv[4][F32_R][4];
            // whole step inside the split and whole 16-byte chunks: plain loads, no per-value selects
            const bool plain = VEC && base + F32_STEP <= re && cb + 24 < chunks && 4 * (cb + 24) + 3 < d;
            if (plain) {
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int r = 0; r < F32_R; ++r) {
                        const float4 t = *reinterpret_cast<const float4 *>(x + (base + r * F32_ROWS + grp) * ldx + 4 * (cb + 8 * i));
                        xv[i][r][0] = t.x; xv[i][r][1] = t.y; xv[i][r][2] = t.z; xv[i][r][3] = t.w;
                    }
            } else
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = cb + 8 * i;
#pragma unroll
                for (int r = 0; r < F32_R; ++r) {
                    const int64_t row = base + r * F32_ROWS + grp;
                    const float *xr = x + row * ldx;
                    if (row >= re || c >= chunks) {
                        xv[i][r][0] = xv[i][r][1] = xv[i][r][2] = xv[i][r][3] = 0.0f;
                    } else if (VEC && 4 * c + 3 < d) {
                        const float4 t = *reinterpret_cast<const float4 *>(xr + 4 * c);
                        xv[i][r][0] = t.x; xv[i][r][1] = t.y; xv[i][r][2] = t.z; xv[i][r][3] = t.w;
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e) xv[i][r][e] = (4 * c + e < d) ? xr[4 * c + e] : 0.0f;
                    }
                }
            }
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int c = cb + 8 * i;
                if (c < chunks) {
#pragma unroll
                    for (int j = 0; j < QT; ++j) {
                        const float4 qq = *reinterpret_cast<const float4 *>(qs + j * dp + 4 * c);
                        const float qa[4] = {qq.x, qq.y, qq.z, qq.w};
#pragma unroll
                        for (int r = 0; r < F32_R; ++r)
#pragma unroll
                            for (int e = 0; e < 4; ++e) {
                                if (l2) { const float t = qa[e] - xv[i][r][e]; acc[j][r] = fmaf(t, t, acc[j][r]); }
                                else acc[j][r] = fmaf(qa[e], xv[i][r][e], acc[j][r]);
                            }
                    }
                }
            }
        }
        // Sum over the 8 lanes of a row group by a halving butterfly: at each step a lane keeps one
        // half of its partial sums and receives the partner's partial sums of that half, so the
        // exchange costs QT * F32_R - 1 shuffles in all (not 3 per sum) and the finished sums end up
        // spread over the lanes: lane `sub` owns sums [sub * PER, sub * PER + PER) in (query, row)
        // order, and tests them against its queries' thresholds.
        constexpr int NACC = QT * F32_R;
        constexpr int PER = NACC >= 8 ? NACC / 8 : 1;
        float red[NACC];
#pragma unroll
        for (int j = 0; j < QT; ++j)
#pragma unroll
            for (int r = 0; r < F32_R; ++r) red[j * F32_R + r] = acc[j][r];
        halve_sums<NACC, DPP_HALF_MIRROR>(red, (sub & 4) != 0);               // partner 7 - sub: bit 2 differs
        halve_sums<(NACC > 1 ? NACC / 2 : 1), DPP_XOR2>(red, (sub & 2) != 0);
        halve_sums<(NACC > 3 ? NACC / 4 : 1), DPP_XOR1>(red, (sub & 1) != 0);
        // NACC >= 8: lane sub holds sums sub * PER + i.  NACC = 4 (one query): after the two halving
        // steps lanes 2p and 2p + 1 both hold sum p; the even lane acts.
        const int first = NACC >= 8 ? sub * PER : (sub >> 1);
        const bool acts = NACC >= 8 || (sub & 1) == 0;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int idx = first + i, j = idx / F32_R, r = idx % F32_R;
            const int64_t row = base + r * F32_ROWS + grp;
            if (acts && row < re) {
                const float a = red[i];
                const cand_t c = make_cand(float_to_sortable(l2 ? a : -a), (uint32_t)row);
                if (c < s_thr[j]) {
                    const int pos = atomicAdd(&s_count[j], 1);
                    buf[(size_t)j * cap + pos] = c;
                }
            }
        }
        __syncthreads();
#pragma unroll
        for (int j = 0; j < QT; ++j) block_compact_if_full(buf + (size_t)j * cap, cap, k, F32_STEP, &s_count[j], &s_thr[j]);
    }
    for (int j = 0; j < QT; ++j) {
        block_bitonic_sort(buf + (size_t)j * cap, cap);
        if (q0 + j < nq) {
            cand_t *out = lists + ((q0 + j) * S + s) * k;
            for (int i = threadIdx.x; i < k; i += F32_THREADS) out[i] = buf[(size_t)j * cap + i];
        }
    }
}

int f32_cap(int k) { return next_pow2((2 * k > k + 2 * F32_STEP) ? 2 * k : k + 2 * F32_STEP); }

// queries per workgroup: as many as fit in 48 KB of LDS with their candidate buffers, at most 8
int f32_query_tile(int d, int k)
{
    const size_t per = (size_t)f32_cap(k) * sizeof(cand_t) + (size_t)((d + 3) / 4) * 16;
    int qt = 8;
    while (qt > 1 && qt * per > 48 * 1024) qt >>= 1;
    return qt;
}

int f32_splits(int64_t n, int64_t nq, int d, int k)
{
    const int64_t tiles = ceil_div(nq > 0 ? nq : 1, f32_query_tile(d, k));
    int64_t s = ceil_div(2048, tiles);
    const int64_t by_rows = n / 2048 > 0 ? n / 2048 : 1;
    if (s > by_rows) s = by_rows;
    if (s > merge_max_lists(k)) s = merge_max_lists(k);
    return (int)(s < 1 ? 1 : s);
}

template <int QT>
hipError_t launch_f32_tile(bool vec, unsigned blocks, size_t shmem, hipStream_t st, const float *x, int64_t n,
                           int64_t ldx, const float *q, int64_t ldq, int64_t nq, int d, int k, int mode, int S,
                           int64_t split_rows, cand_t *lists, int cap)
{
    const bool l2 = mode == MODE_F32_L2;
    auto kern = vec ? (l2 ? search_f32_kernel<true, QT, true> : search_f32_kernel<true, QT, false>)
                    : (l2 ? search_f32_kernel<false, QT, true> : search_f32_kernel<false, QT, false>);
    kern<<<blocks, F32_THREADS, shmem, st>>>(x, n, ldx, q, ldq, nq, d, k, mode, S, split_rows, lists, cap);
    return hipGetLastError();
}

}  // namespace

// Largest d a search for k results takes: one query's vector and candidate buffer, plus the kernel's
// 96 bytes of static LDS, must fit the 64 KB a workgroup may use without opting in to more.
int f32_max_d(int k)
{
    const int64_t room = 64 * 1024 - 128 - (int64_t)f32_cap(k) * (int64_t)sizeof(cand_t);
    return room < 16 ? 0 : (int)(room / 16 * 4);
}

size_t f32_workspace_bytes(int64_t n, int64_t nq, int d, int k)
{
    return (size_t)nq * f32_splits(n, nq, d, k) * k * sizeof(cand_t);
}

hipError_t launch_search_f32(const float *x, int64_t n, int64_t ldx, const float *q, int64_t nq, int64_t ldq,
                             int d, int k, int metric, int32_t *ids, float *dists, void *ws, hipStream_t st)
{
    const int S = f32_splits(n, nq, d, k);
    const int qt = f32_query_tile(d, k);
    const int mode = metric == LPQ_METRIC_L2SQ ? MODE_F32_L2 : MODE_F32_IP;
    const int cap = f32_cap(k);
    const int64_t split_rows = round_up(ceil_div(n, S), F32_STEP);
    const size_t shmem = (size_t)qt * ((size_t)cap * sizeof(cand_t) + (size_t)((d + 3) / 4) * 16);
    if (d > f32_max_d(k) || shmem + 128 > 64 * 1024) return hipErrorInvalidValue;   // callers check f32_max_d first
    cand_t *lists = reinterpret_cast<cand_t *>(ws);
    const bool vec = ((uintptr_t)x % 16 == 0) && (ldx % 4 == 0);
    const unsigned blocks = (unsigned)(ceil_div(nq, qt) * S);
    hipError_t e;
    switch (qt) {
    case 8: e = launch_f32_tile<8>(vec, blocks, shmem, st, x, n, ldx, q, ldq, nq, d, k, mode, S, split_rows, lists, cap); break;
    case 4: e = launch_f32_tile<4>(vec, blocks, shmem, st, x, n, ldx, q, ldq, nq, d, k, mode, S, split_rows, lists, cap); break;
    case 2: e = launch_f32_tile<2>(vec, blocks, shmem, st, x, n, ldx, q, ldq, nq, d, k, mode, S, split_rows, lists, cap); break;
    default: e = launch_f32_tile<1>(vec, blocks, shmem, st, x, n, ldx, q, ldq, nq, d, k, mode, S, split_rows, lists, cap); break;
    }
    if (e != hipSuccess) return e;
    return launch_merge(lists, nq, S, k, nullptr, nullptr, nullptr, ids, reinterpret_cast<int32_t *>(dists),
                        nullptr, mode, st, true);
}

}  // namespace lpq
