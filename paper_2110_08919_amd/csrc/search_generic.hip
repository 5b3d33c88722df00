// Generic integer search kernel: any padded dimension, any k <= MAX_K.  One workgroup scans
// one corpus split for one query with 4-way int8 dot products, keeps the candidates that
// beat the running k-th best in an LDS buffer and compacts the buffer by a bitonic sort
// whenever it could overflow.  It is the fallback for shapes the matrix-core kernel does
// not take and an independent second implementation of the same result.
#include <type_traits>

#include "block_select.h"
#include "lpq_internal.h"
#include "wave_ops.h"

namespace lpq {

namespace {

constexpr int GEN_THREADS = 256;
constexpr int GEN_ROWS = GEN_THREADS / 8;  // rows per step: 8 lanes share a row

// One (query, corpus split) pair by the whole workgroup; must be reached by all its threads.
__device__ __forceinline__ void generic_scan(const SearchArgs &a, int64_t rs, int64_t re, int64_t q, const cand_t *seeds,
                                             cand_t *out, int cap, cand_t *buf, uint4 *qs, int *s_count, cand_t *s_thr)
{
    const int chunks = a.d_pad >> 4;  // 16-byte chunks per row of int8 codes
    const bool l2 = a.metric == LPQ_METRIC_L2SQ;
    for (int c = threadIdx.x; c < chunks; c += GEN_THREADS)
        qs[c] = reinterpret_cast<const uint4 *>(a.qcodes + q * a.d_pad)[c];
    // Packed rows: a 16-byte chunk holds 32 codes, two to a byte, stored + 8; the low nibbles of a
    // dword meet one dword of the (permuted) query codes and its high nibbles the next one, as in
    // the matrix-core scan.  The result is dot(code + 8, q): the same key that scan produces.
    const int xchunks = a.packed ? chunks >> 1 : chunks;
    const int64_t row_bytes = a.packed ? a.d_pad >> 1 : a.d_pad;
    for (int i = threadIdx.x; i < cap; i += GEN_THREADS) buf[i] = CAND_NONE;
    if (threadIdx.x == 0) {
        *s_count = 0;
        *s_thr = seeds ? seeds[q] : CAND_NONE;
    }
    __syncthreads();

    const int sub = threadIdx.x & 7, grp = threadIdx.x >> 3;
    for (int64_t base = rs; base < re; base += GEN_ROWS) {
        const int64_t row = base + grp;
        int dot = 0;
        if (row < re) {
            const uint4 *xr = reinterpret_cast<const uint4 *>(a.codes + row * row_bytes);
            if (a.packed) {
                for (int c = sub; c < xchunks; c += 8) {
                    const uint4 xv = xr[c], q0 = qs[2 * c], q1 = qs[2 * c + 1];
                    const unsigned m = 0x0F0F0F0Fu;
                    dot = __builtin_amdgcn_sdot4((int)(xv.x & m), (int)q0.x, dot, false);
                    dot = __builtin_amdgcn_sdot4((int)((xv.x >> 4) & m), (int)q0.y, dot, false);
                    dot = __builtin_amdgcn_sdot4((int)(xv.y & m), (int)q0.z, dot, false);
                    dot = __builtin_amdgcn_sdot4((int)((xv.y >> 4) & m), (int)q0.w, dot, false);
                    dot = __builtin_amdgcn_sdot4((int)(xv.z & m), (int)q1.x, dot, false);
                    dot = __builtin_amdgcn_sdot4((int)((xv.z >> 4) & m), (int)q1.y, dot, false);
                    dot = __builtin_amdgcn_sdot4((int)(xv.w & m), (int)q1.z, dot, false);
                    dot = __builtin_amdgcn_sdot4((int)((xv.w >> 4) & m), (int)q1.w, dot, false);
                }
            } else {
                for (int c = sub; c < chunks; c += 8) {
                    const uint4 xv = xr[c], qv = qs[c];
                    dot = __builtin_amdgcn_sdot4((int)xv.x, (int)qv.x, dot, false);
                    dot = __builtin_amdgcn_sdot4((int)xv.y, (int)qv.y, dot, false);
                    dot = __builtin_amdgcn_sdot4((int)xv.z, (int)qv.z, dot, false);
                    dot = __builtin_amdgcn_sdot4((int)xv.w, (int)qv.w, dot, false);
                }
            }
        }
        dot += __shfl_xor(dot, 4, 64);
        dot += __shfl_xor(dot, 2, 64);
        dot += __shfl_xor(dot, 1, 64);
        if (sub == 0 && row < re) {
            const int32_t key = (l2 ? a.norms[row] : 0) - 2 * dot;  // see cand_t
            const cand_t c = make_cand(key, (uint32_t)row);
            if (c < *s_thr) {
                const int pos = atomicAdd(s_count, 1);
                buf[pos] = c;
            }
        }
        __syncthreads();
        block_compact_if_full(buf, cap, a.k, GEN_ROWS, s_count, s_thr);
    }
    block_bitonic_sort(buf, cap);
    for (int i = threadIdx.x; i < a.k; i += GEN_THREADS) out[i] = buf[i];
    __syncthreads();   // buf and qs are free again
}

__global__ __launch_bounds__(GEN_THREADS) void search_generic_kernel(
    SearchArgs a, int64_t row0, int64_t row1, int S, int64_t split_rows, const cand_t *__restrict__ seeds,
    cand_t *__restrict__ lists, int cap)
{
    extern __shared__ __align__(16) unsigned char smem[];
    cand_t *buf = reinterpret_cast<cand_t *>(smem);
    uint4 *qs = reinterpret_cast<uint4 *>(buf + cap);
    __shared__ int s_count;
    __shared__ cand_t s_thr;
    const int64_t q = blockIdx.x / S;
    const int s = blockIdx.x % S;
    const int64_t rs = row0 + (int64_t)s * split_rows;
    const int64_t re = (rs + split_rows < row1) ? rs + split_rows : row1;
    generic_scan(a, rs, re, q, seeds, lists + ((int64_t)q * S + s) * a.k, cap, buf, qs, &s_count, &s_thr);
}

// The same scan for a LIST of queries (the ones a collecting scan could not finish): the
// workgroups of a fixed-size grid share out the (listed query, split) pairs, so a handful of
// queries is spread over the whole chip and an empty list costs one tiny launch.
__global__ __launch_bounds__(GEN_THREADS) void search_generic_list_kernel(
    SearchArgs a, int64_t row0, int64_t row1, int S, int64_t split_rows, const int32_t *__restrict__ qlist,
    const int32_t *__restrict__ qcount, cand_t *__restrict__ lists, int cap, int max_listed)
{
    extern __shared__ __align__(16) unsigned char smem[];
    cand_t *buf = reinterpret_cast<cand_t *>(smem);
    uint4 *qs = reinterpret_cast<uint4 *>(buf + cap);
    __shared__ int s_count;
    __shared__ cand_t s_thr;
    if (*qcount > max_listed) return;                       // too many for this path: another kernel takes them
    const int64_t items = (int64_t)(*qcount) * S;           // same for every thread of the grid
    for (int64_t item = blockIdx.x; item < items; item += gridDim.x) {
        const int64_t q = qlist[item / S];
        const int s = (int)(item % S);
        const int64_t rs = row0 + (int64_t)s * split_rows;
        const int64_t re = (rs + split_rows < row1) ? rs + split_rows : row1;
        generic_scan(a, rs, re, q, nullptr, lists + ((int64_t)q * S + s) * a.k, cap, buf, qs, &s_count, &s_thr);
    }
}

// 64-bit minimum over the wave; every lane gets the result.
__device__ __forceinline__ cand_t wave_min_cand(cand_t c) { return wave_min_u64(c); }

// Final id and distance of candidate c of query q, written at position `at`.
__device__ __forceinline__ void emit_result(cand_t c, int64_t at, int64_t q, int32_t *__restrict__ ids,
                                            int32_t *__restrict__ dists, const int32_t *__restrict__ qnorms, int metric)
{
    const int32_t key = cand_key(c);
    ids[at] = (c == CAND_NONE) ? -1 : (int32_t)cand_id(c);
    int32_t v;
    if (metric == MODE_I8_L2) v = key + qnorms[q];
    else if (metric == MODE_I8_IP) v = -(key / 2);
    else if (metric == MODE_I8_IP_ADJ) v = -(key / 2) + qnorms[q];
    else {
        const float f = sortable_to_float(key);
        v = __float_as_int(metric == MODE_F32_L2 ? f : -f);
    }
    dists[at] = v;
}

// One workgroup per query: sort all candidates of its P lists (plus an optional extra list).
__global__ __launch_bounds__(256) void merge_kernel(
    const cand_t *__restrict__ lists, int P, int k, const cand_t *__restrict__ extra, int cap,
    cand_t *__restrict__ out_lists, cand_t *__restrict__ seeds_out, int32_t *__restrict__ ids,
    int32_t *__restrict__ dists, const int32_t *__restrict__ qnorms, int metric, const int32_t *__restrict__ only,
    const int32_t *__restrict__ gate_count, int gate_lo, int gate_hi)
{
    extern __shared__ __align__(16) unsigned char smem[];
    cand_t *buf = reinterpret_cast<cand_t *>(smem);
    const int64_t q = blockIdx.x;
    if (only && !only[q]) return;   // same for the whole workgroup
    if (gate_count) {               // this merge belongs to one of two alternative redo paths
        const int c = *gate_count;
        if (c < gate_lo || c > gate_hi) return;
    }
    const int m = P * k;
    for (int i = threadIdx.x; i < cap; i += 256) {
        cand_t c = CAND_NONE;
        if (i < m) c = lists[q * m + i];
        else if (extra && i < m + k) c = extra[q * k + (i - m)];
        buf[i] = c;
    }
    __syncthreads();
    block_bitonic_sort(buf, cap);
    for (int i = threadIdx.x; i < k; i += 256) {
        const cand_t c = buf[i];
        if (out_lists) out_lists[q * k + i] = c;
        if (ids) emit_result(c, q * k + i, q, ids, dists, qnorms, metric);
    }
    if (seeds_out && threadIdx.x == 0) seeds_out[q] = buf[k - 1];
}

// Last step of the collecting scan for small k (<= 32) and at most 64 regions, one WAVE per query
// and no LDS: lane r owns region r.  In each pass every lane loads up to 8 more candidates of its
// region into registers; together with the k best kept so far (lane i keeps the i-th best) the
// wave takes the smallest k times, which become the kept ones of the next pass.  Any number of
// candidates the regions can hold is handled; a query with an overflowed region or fewer than k
// candidates is flagged in over[] instead.
__global__ __launch_bounds__(256) void collect_select_wave_kernel(
    const cand_t *__restrict__ cbuf, const int32_t *__restrict__ ccnt, int64_t nq, int SS, int Cs, int k,
    int32_t *__restrict__ over, int32_t *__restrict__ qlist, int32_t *__restrict__ qcount,
    int32_t *__restrict__ ids, int32_t *__restrict__ dists, const int32_t *__restrict__ qnorms, int metric)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t q = (int64_t)blockIdx.x * 4 + wave;
    if (q >= nq) return;                                   // wave-uniform
    const int c = (lane < SS) ? ccnt[q * SS + lane] : 0;
    const bool bad = c > Cs || c < 0;
    int total = bad ? 0 : c, most = total;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) {
        total += __shfl_xor(total, o, 64);
        const int t = __shfl_xor(most, o, 64);
        most = t > most ? t : most;
    }
    if (__ballot(bad) || total < k) {
        if (lane == 0) { over[q] = 1; qlist[atomicAdd(qcount, 1)] = (int32_t)q; }
        return;
    }
    const cand_t *mine = cbuf + ((size_t)q * SS + (lane < SS ? lane : 0)) * Cs;
    cand_t keep = CAND_NONE;                               // lane i: the i-th best so far
    constexpr int E = 8;                                   // candidates a lane takes per pass
    for (int p0 = 0; p0 < most; p0 += E) {                 // wave-uniform trip count
        cand_t v[E + 1];
#pragma unroll
        for (int e = 0; e < E; ++e) v[e] = (p0 + e < c && !bad) ? mine[p0 + e] : CAND_NONE;
        v[E] = keep;
        cand_t next = CAND_NONE;
        for (int r = 0; r < k; ++r) {
            cand_t m = v[0];
#pragma unroll
            for (int e = 1; e <= E; ++e) m = v[e] < m ? v[e] : m;
            const cand_t mn = wave_min_cand(m);
            if (lane == r) next = mn;
            const int win = __ffsll((unsigned long long)__ballot(m == mn)) - 1;
            bool done = lane != win || mn == CAND_NONE;
#pragma unroll
            for (int e = 0; e <= E; ++e) {
                const bool hit = !done && v[e] == mn;
                v[e] = hit ? CAND_NONE : v[e];
                done = done || hit;
            }
        }
        keep = next;
    }
    if (lane < k) emit_result(keep, q * k + lane, q, ids, dists, qnorms, metric);
    if (lane == 0) over[q] = 0;
}

// 64-bit value of lane `src` (any lane), through two 32-bit shuffles.
__device__ __forceinline__ cand_t shfl_u64(cand_t v, int src)
{
    const unsigned lo = (unsigned)__shfl((int)(uint32_t)v, src, 64), hi = (unsigned)__shfl((int)(uint32_t)(v >> 32), src, 64);
    return ((cand_t)hi << 32) | lo;
}

// Ascending bitonic sort of 64 E candidates held E per lane by one wave, element e = E * lane + slot.
// Strides below E exchange registers of a lane, larger strides exchange with lane ^ (stride / E).
template <int E>
__device__ __forceinline__ void wave_sort(cand_t (&v)[E], int lane)
{
#pragma unroll
    for (int size = 2; size <= 64 * E; size <<= 1) {
#pragma unroll
        for (int stride = size >> 1; stride >= 1; stride >>= 1) {
            if (stride >= E) {
                const int lx = stride / E;
                const bool up = ((lane * E) & size) == 0;          // this run of `size` elements sorts ascending
                const bool low = (lane & lx) == 0;                 // this lane holds the lower element of each pair
                const bool take_min = up == low;
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    const cand_t o = shfl_u64(v[j], lane ^ lx);
                    v[j] = take_min ? (o < v[j] ? o : v[j]) : (o > v[j] ? o : v[j]);
                }
            } else {
#pragma unroll
                for (int j = 0; j < E; ++j) {
                    if ((j & stride) == 0) {
                        const bool up = ((lane * E + j) & size) == 0;
                        const cand_t a = v[j], b = v[j | stride];
                        const bool swap = up ? (b < a) : (a < b);
                        v[j] = swap ? b : a;
                        v[j | stride] = swap ? a : b;
                    }
                }
            }
        }
    }
}

// Last step of the collecting scan for k <= 128 and at most 64 regions, one WAVE per query and no
// LDS: lane r holds the count of region r; the wave loads up to 512 candidates (2, 4 or 8 per lane
// as needed, each found by a search over the prefix counts), sorts them in registers and keeps the
// best 128 in its first 16 lanes; further candidates come in 384 at a time through the other 48 lanes.  Any number
// of candidates the regions hold is handled; a query with an overflowed region or fewer than k
// candidates is flagged in over[] instead.
__global__ __launch_bounds__(256) void collect_select_sort_kernel(
    const cand_t *__restrict__ cbuf, const int32_t *__restrict__ ccnt, int64_t nq, int SS, int Cs, int k,
    int32_t *__restrict__ over, int32_t *__restrict__ qlist, int32_t *__restrict__ qcount,
    int32_t *__restrict__ ids, int32_t *__restrict__ dists, const int32_t *__restrict__ qnorms, int metric)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t q = (int64_t)blockIdx.x * 4 + wave;
    if (q >= nq) return;                                   // wave-uniform
    const int c = (lane < SS) ? ccnt[q * SS + lane] : 0;
    const bool bad = c > Cs || c < 0;
    int incl = bad ? 0 : c;                                // inclusive prefix sum of the counts over the lanes
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const int t = __shfl_up(incl, o, 64);
        if (lane >= o) incl += t;
    }
    const int total = __shfl(incl, 63, 64);
    if (__ballot(bad) || total < k) {
        if (lane == 0) { over[q] = 1; qlist[atomicAdd(qcount, 1)] = (int32_t)q; }
        return;
    }
    const int excl = incl - c;                             // index of the first candidate of this lane's region
    const cand_t *base = cbuf + (size_t)q * SS * Cs;
    // candidate number i of the query sits in the first region whose inclusive count exceeds i
    auto fetch = [&](int i) -> cand_t {
        int r = 0;
#pragma unroll
        for (int step = 32; step >= 1; step >>= 1)
            if (__shfl(incl, r + step - 1, 64) <= i) r += step;
        r = r > 63 ? 63 : r;
        const int first = __shfl(excl, r, 64);
        return i < total ? base[(size_t)r * Cs + (i - first)] : CAND_NONE;
    };
    // few candidates: a smaller network (2 or 4 per lane) does
    auto small = [&](auto tag) {
        constexpr int E = decltype(tag)::value;
        cand_t v[E];
#pragma unroll
        for (int j = 0; j < E; ++j) v[j] = fetch(j * 64 + lane);
        wave_sort<E>(v, lane);
#pragma unroll
        for (int j = 0; j < E; ++j) {
            const int e = lane * E + j;
            if (e < k) emit_result(v[j], q * k + e, q, ids, dists, qnorms, metric);
        }
    };
    if (total <= 128) {                                    // wave-uniform
        small(std::integral_constant<int, 2>{});
    } else if (total <= 256) {
        small(std::integral_constant<int, 4>{});
    } else {
        cand_t v[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) v[j] = fetch(j * 64 + lane);
        wave_sort<8>(v, lane);
        for (int done = 512; done < total; done += 384) {  // wave-uniform: the best 128 stay in lanes 0 .. 15
#pragma unroll
            for (int j = 0; j < 8; ++j) {
                const cand_t n = fetch(done + j * 48 + (lane - 16));   // (every lane takes part in the shuffles)
                if (lane >= 16) v[j] = n;
            }
            wave_sort<8>(v, lane);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
            const int e = lane * 8 + j;
            if (e < k) emit_result(v[j], q * k + e, q, ids, dists, qnorms, metric);
        }
    }
    if (lane == 0) over[q] = 0;
}

// Last step of the collecting scan, one workgroup per query: gather the query's regions into LDS,
// sort, write the k best.  A query with an overflowed region, more than `maxc` candidates or fewer
// than k is flagged in over[] instead and left to the generic kernel.
__global__ __launch_bounds__(256) void collect_select_kernel(
    const cand_t *__restrict__ cbuf, const int32_t *__restrict__ ccnt, int SS, int Cs, int k, int maxc,
    int32_t *__restrict__ over, int32_t *__restrict__ qlist, int32_t *__restrict__ qcount,
    int32_t *__restrict__ ids, int32_t *__restrict__ dists, const int32_t *__restrict__ qnorms, int metric,
    const int32_t *__restrict__ only, const int32_t *__restrict__ gate_count, int gate_min)
{
    extern __shared__ __align__(16) unsigned char smem[];
    cand_t *buf = reinterpret_cast<cand_t *>(smem);            // [maxc]
    int *off = reinterpret_cast<int *>(buf + maxc);            // [SS + 1] first slot of each region
    __shared__ int tsum[256];
    __shared__ int s_bad;
    const int64_t q = blockIdx.x;
    const int tid = threadIdx.x;
    if (only) {   // second round: queries flagged in the first one, if they were more than gate_min
        if (*gate_count <= gate_min || !only[q]) {
            if (tid == 0) over[q] = 0;
            return;
        }
    }
    const int per = (SS + 255) / 256;                          // consecutive regions per thread
    const int r0 = tid * per, r1 = (r0 + per < SS) ? r0 + per : SS;
    if (tid == 0) s_bad = 0;
    __syncthreads();
    int local = 0;
    bool bad = false;
    for (int r = r0; r < r1; ++r) {
        const int c = ccnt[q * SS + r];
        bad |= c > Cs || c < 0;
        local += (c > Cs) ? Cs : (c < 0 ? 0 : c);
    }
    if (bad) s_bad = 1;
    tsum[tid] = local;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {                        // inclusive scan of the thread sums
        const int v = (tid >= o) ? tsum[tid - o] : 0;
        __syncthreads();
        tsum[tid] += v;
        __syncthreads();
    }
    const int M = tsum[255];
    if (s_bad || M > maxc || M < k) {
        if (tid == 0) { over[q] = 1; qlist[atomicAdd(qcount, 1)] = (int32_t)q; }
        return;
    }
    int run = tsum[tid] - local;
    for (int r = r0; r < r1; ++r) {
        off[r] = run;
        const int c = ccnt[q * SS + r];
        run += c;
    }
    if (tid == 255) off[SS] = M;
    const int cap = next_pow2(M < 2 ? 2 : M);
    __syncthreads();
    for (int i = tid; i < cap; i += 256) {
        cand_t c = CAND_NONE;
        if (i < M) {
            int lo = 0, hi = SS;                               // last region with off[r] <= i
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (off[mid] <= i) lo = mid; else hi = mid;
            }
            c = cbuf[((size_t)q * SS + lo) * Cs + (i - off[lo])];
        }
        buf[i] = c;
    }
    __syncthreads();
    block_bitonic_sort(buf, cap);
    for (int i = tid; i < k; i += 256) emit_result(buf[i], q * k + i, q, ids, dists, qnorms, metric);
    if (tid == 0) over[q] = 0;
}

// Tighter bounds for queries whose regions overflowed.  Whatever the scan did collect for such a
// query are real items, so the k-th best of them bounds the query's final k-th best from above -
// and far more closely than the seeding pass did, since they all passed its bound.  One workgroup
// per query: every region gives its first min(count, Cs, maxc / SS) candidates, the workgroup
// sorts them and writes bounds_out[q] = the candidate right after the k-th best in (key, id)
// order: the k-th best and everything before it pass, so ties of its key with larger ids do not
// (a region keeps its FIRST arrivals, the lowest ids among equal keys, which is what makes this
// converge on codes of few bits).  With fewer than k collected the old bound is kept.  Queries that are
// not flagged get the bound nothing passes (candidate 0), and so does every query when no more
// than min_flagged are flagged (then the second scan does not run at all).  Also clears *zero_word.
__global__ __launch_bounds__(256) void collect_refine_kernel(
    const cand_t *__restrict__ cbuf, const int32_t *__restrict__ ccnt, int SS, int Cs, int k, int maxc,
    const int32_t *__restrict__ over, const int32_t *__restrict__ qcount, int min_flagged,
    const cand_t *bounds_in, cand_t *bounds_out /* may be the same array */, int32_t *__restrict__ zero_word)
{
    extern __shared__ __align__(16) unsigned char smem[];
    cand_t *buf = reinterpret_cast<cand_t *>(smem);            // [maxc]
    const int64_t q = blockIdx.x;
    const int tid = threadIdx.x;
    if (q == 0 && tid == 0 && zero_word) *zero_word = 0;
    if (*qcount <= min_flagged || !over[q]) {
        if (tid == 0) bounds_out[q] = 0;
        return;
    }
    const int per = maxc / SS < Cs ? maxc / SS : Cs;           // slots per region, >= 1
    const int used = SS * per;
    const int cap = next_pow2(used < 2 ? 2 : used);
    for (int i = tid; i < cap; i += 256) {
        cand_t c = CAND_NONE;
        if (i < used) {
            const int r = i / per, j = i - r * per;
            const int cnt = ccnt[q * SS + r];
            if (j < cnt) c = cbuf[((size_t)q * SS + r) * Cs + j];   // cnt > Cs: the region holds Cs, and j < per <= Cs
        }
        buf[i] = c;
    }
    __syncthreads();
    block_bitonic_sort(buf, cap);
    cand_t kth = (k <= cap) ? buf[k - 1] : CAND_NONE;   // the same value in every thread
    __syncthreads();
    // Second pass when the regions hold more than the sort does (per < Cs): every collected
    // candidate that is no worse than that k-th best goes into the buffer - about k Cs / per of
    // them - and the k-th best of ALL collected candidates comes out.  (If even those do not fit,
    // the first estimate stands: it is a valid bound either way.)
    if (per < Cs && kth != CAND_NONE) {
        __shared__ int s_n;
        if (tid == 0) s_n = 0;
        __syncthreads();
        for (int r = 0; r < SS; ++r) {
            int cnt = ccnt[q * SS + r];
            cnt = cnt > Cs ? Cs : cnt;
            for (int j = tid; j < cnt; j += 256) {
                const cand_t c = cbuf[((size_t)q * SS + r) * Cs + j];
                if (c <= kth) {
                    const int at = atomicAdd(&s_n, 1);
                    if (at < maxc) buf[at] = c;
                }
            }
        }
        __syncthreads();
        const int m = s_n;
        if (m >= k && m <= maxc) {
            const int cap2 = next_pow2(m < 2 ? 2 : m);
            for (int i = m + tid; i < cap2; i += 256) buf[i] = CAND_NONE;
            __syncthreads();
            block_bitonic_sort(buf, cap2);
            kth = buf[k - 1];
        }
    }
    // the scan passes candidates strictly below its bound: kth itself must pass, later ids with its key need not
    if (tid == 0) bounds_out[q] = (kth == CAND_NONE) ? bounds_in[q] : kth + 1;
}

// Merge of lists that are each sorted ascending, for small k and many lists: one workgroup per
// query; every wave takes k times the smallest head among its share of the lists (each lane owns
// the lists first + lane, first + lane + 64, ...), then wave 0 does the same over the four wave
// results.  Duplicated values come out once per copy, as a sort would give them.
// A lane keeps the head and the position of each of its LPL lists in registers, so a round costs the
// winner one LDS read (the next entry of the list it took from) instead of a walk over positions and
// heads in LDS (512 lists of 10: 16.9 -> see the profile of the small-batch workload).
template <int LPL>
__global__ __launch_bounds__(256) void merge_sorted_kernel(
    const cand_t *__restrict__ lists, int P, int k, const cand_t *__restrict__ extra,
    cand_t *__restrict__ out_lists, cand_t *__restrict__ seeds_out, int32_t *__restrict__ ids,
    int32_t *__restrict__ dists, const int32_t *__restrict__ qnorms, int metric)
{
    extern __shared__ __align__(16) unsigned char smem[];
    const int Pt = P + (extra ? 1 : 0);
    cand_t *buf = reinterpret_cast<cand_t *>(smem);     // [Pt][k]
    cand_t *wres = buf + (size_t)Pt * k;                // [4][k]
    const int64_t q = blockIdx.x;
    const int m = P * k, mt = Pt * k;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (int i = threadIdx.x; i < mt; i += 256) buf[i] = (i < m) ? lists[q * m + i] : extra[q * k + (i - m)];
    __syncthreads();

    const int lpw = (Pt + 3) >> 2;                      // lists per wave, <= 64 LPL
    const int first = wave * lpw, last = (first + lpw < Pt) ? first + lpw : Pt;
    cand_t head[LPL];
    int pos[LPL];
#pragma unroll
    for (int j = 0; j < LPL; ++j) {
        const int l = first + lane + 64 * j;
        pos[j] = 0;
        head[j] = (l < last) ? buf[(size_t)l * k] : CAND_NONE;
    }
    for (int r = 0; r < k; ++r) {
        cand_t best = head[0];
#pragma unroll
        for (int j = 1; j < LPL; ++j) best = head[j] < best ? head[j] : best;
        const cand_t mn = wave_min_cand(best);
        const int win = __ffsll((unsigned long long)__ballot(best == mn)) - 1;
        if (lane == win) {
            wres[wave * k + r] = mn;
            if (mn != CAND_NONE) {
                bool taken = false;                     // the first of my lists whose head is the minimum moves on
#pragma unroll
                for (int j = 0; j < LPL; ++j) {
                    if (!taken && head[j] == mn) {
                        taken = true;
                        pos[j] += 1;
                        head[j] = (pos[j] < k) ? buf[(size_t)(first + lane + 64 * j) * k + pos[j]] : CAND_NONE;
                    }
                }
            }
        }
    }
    __syncthreads();
    if (wave != 0) return;
    int p2 = 0;
    cand_t best = (lane < 4) ? wres[lane * k] : CAND_NONE;
    for (int r = 0; r < k; ++r) {
        const cand_t mn = wave_min_cand(best);
        const int win = __ffsll((unsigned long long)__ballot(best == mn)) - 1;
        if (lane == win) {
            if (out_lists) out_lists[q * k + r] = mn;
            if (seeds_out && r == k - 1) seeds_out[q] = mn;
            if (ids) emit_result(mn, q * k + r, q, ids, dists, qnorms, metric);
            if (lane < 4 && mn != CAND_NONE) {
                ++p2;
                best = (p2 < k) ? wres[lane * k + p2] : CAND_NONE;
            }
        }
    }
}

// One workgroup per (query, group): sort the candidates of `group` consecutive lists.
__global__ __launch_bounds__(256) void merge_groups_kernel(const cand_t *__restrict__ lists, int P, int group, int groups,
                                                           int k, int cap, cand_t *__restrict__ out_lists)
{
    extern __shared__ __align__(16) unsigned char smem[];
    cand_t *buf = reinterpret_cast<cand_t *>(smem);
    const int64_t q = blockIdx.x / groups;
    const int g = blockIdx.x % groups;
    const int first = g * group, count = (first + group <= P ? group : P - first) * k;
    for (int i = threadIdx.x; i < cap; i += 256) buf[i] = (i < count) ? lists[(q * P + first) * k + i] : CAND_NONE;
    __syncthreads();
    block_bitonic_sort(buf, cap);
    for (int i = threadIdx.x; i < k; i += 256) out_lists[(q * groups + g) * k + i] = buf[i];
}

}  // namespace

hipError_t launch_merge_groups(const cand_t *lists, int64_t nq, int P, int group, int k, cand_t *out_lists,
                               hipStream_t st)
{
    if (nq <= 0) return hipSuccess;
    const int groups = (int)ceil_div(P, group);
    const int cap = next_pow2(group * k < 2 ? 2 : group * k);
    if (cap > 4096) return hipErrorInvalidValue;
    merge_groups_kernel<<<(unsigned)(nq * groups), 256, (size_t)cap * sizeof(cand_t), st>>>(lists, P, group, groups, k,
                                                                                          cap, out_lists);
    return hipGetLastError();
}

namespace {
}  // namespace

int merge_max_lists(int k) { return 4096 / k - 1; }

// Lists of k that are each sorted and short (k <= 32) merge by repeated extraction, which needs
// no power-of-two buffer: as many lists as 128 KB of LDS hold, at most 1024.
static size_t merge_sorted_lds(int lists, int k) { return (size_t)(lists + 4) * k * sizeof(cand_t); }
int merge_max_sorted_lists(int k)
{
    if (k > 32) return merge_max_lists(k);
    int p = (int)((131072 - 32 * (size_t)k) / (8 * (size_t)k + 4)) - 1;   // one spare for an extra list
    return p > 1024 ? 1024 : p;
}

hipError_t launch_collect_refine(const cand_t *cbuf, const int32_t *ccnt, int64_t nq, int SS, int Cs, int k,
                                 const int32_t *over, const int32_t *qcount, int min_flagged, const cand_t *bounds_in,
                                 cand_t *bounds_out, int32_t *zero_word, hipStream_t st)
{
    if (nq <= 0) return hipSuccess;
    const int maxc = 4096;
    if (SS < 1 || SS > 2048 || Cs < 1 || k > maxc) return hipErrorInvalidValue;
    collect_refine_kernel<<<(unsigned)nq, 256, (size_t)maxc * sizeof(cand_t), st>>>(cbuf, ccnt, SS, Cs, k, maxc, over, qcount,
                                                                                   min_flagged, bounds_in, bounds_out, zero_word);
    return hipGetLastError();
}

hipError_t launch_collect_select(const cand_t *cbuf, const int32_t *ccnt, int64_t nq, int SS, int Cs, int k,
                                 int32_t *over, int32_t *qlist, int32_t *qcount, int32_t *ids, int32_t *dists,
                                 const int32_t *qnorms, int metric, hipStream_t st, int expected_candidates,
                                 const int32_t *only, const int32_t *gate_count, int gate_min)
{
    if (nq <= 0) return hipSuccess;
    const int maxc = 4096;
    if (SS < 1 || SS > 2048 || k > maxc) return hipErrorInvalidValue;
    // (k rounds of "smallest in the wave" beat the sorting network only for the shortest lists: k = 1
    // 1.00 against 1.01 ms per search on the benchmark workload, k = 10 1.178 against 1.166, k = 32 1.446 against 1.375)
    if (!only && expected_candidates > 0 && expected_candidates <= 256 && SS <= 64 && k <= 2) {
        collect_select_wave_kernel<<<(unsigned)ceil_div(nq, (int64_t)4), 256, 0, st>>>(cbuf, ccnt, nq, SS, Cs, k, over, qlist,
                                                                                 qcount, ids, dists, qnorms, metric);
        return hipGetLastError();
    }
    if (!only && SS <= 64 && k <= 128) {   // one wave per query, sorted in registers
        collect_select_sort_kernel<<<(unsigned)ceil_div(nq, (int64_t)4), 256, 0, st>>>(cbuf, ccnt, nq, SS, Cs, k, over, qlist,
                                                                                 qcount, ids, dists, qnorms, metric);
        return hipGetLastError();
    }
    const size_t lds = (size_t)maxc * sizeof(cand_t) + (size_t)(SS + 1) * sizeof(int);
    collect_select_kernel<<<(unsigned)nq, 256, lds, st>>>(cbuf, ccnt, SS, Cs, k, maxc, over, qlist, qcount, ids, dists,
                                                          qnorms, metric, only, gate_count, gate_min);
    return hipGetLastError();
}

hipError_t launch_search_generic(const SearchArgs &a, int64_t row0, int64_t row1, int S, const cand_t *seeds,
                                 cand_t *lists, hipStream_t st)
{
    if (a.nq <= 0 || row1 <= row0) return hipSuccess;
    const int cap = next_pow2((2 * a.k > a.k + 2 * GEN_ROWS) ? 2 * a.k : a.k + 2 * GEN_ROWS);
    const int64_t split_rows = round_up(ceil_div(row1 - row0, S), GEN_ROWS);
    const size_t shmem = (size_t)cap * sizeof(cand_t) + (size_t)a.d_pad;
    search_generic_kernel<<<(unsigned)(a.nq * S), GEN_THREADS, shmem, st>>>(a, row0, row1, S, split_rows,
                                                                              seeds, lists, cap);
    return hipGetLastError();
}

hipError_t launch_search_generic_list(const SearchArgs &a, int64_t row0, int64_t row1, int S, const int32_t *qlist,
                                      const int32_t *qcount, cand_t *lists, hipStream_t st, int max_listed)
{
    if (a.nq <= 0 || row1 <= row0) return hipSuccess;
    const int cap = next_pow2((2 * a.k > a.k + 2 * GEN_ROWS) ? 2 * a.k : a.k + 2 * GEN_ROWS);
    const int64_t split_rows = round_up(ceil_div(row1 - row0, S), GEN_ROWS);
    const size_t shmem = (size_t)cap * sizeof(cand_t) + (size_t)a.d_pad;
    search_generic_list_kernel<<<2048, GEN_THREADS, shmem, st>>>(a, row0, row1, S, split_rows, qlist, qcount, lists, cap,
                                                                 max_listed);
    return hipGetLastError();
}

hipError_t launch_merge(const cand_t *lists, int64_t nq, int P, int k, const cand_t *extra_lists,
                        cand_t *out_lists, cand_t *seeds_out, int32_t *ids, int32_t *dists,
                        const int32_t *qnorms, int metric, hipStream_t st, bool sorted_lists, const int32_t *only,
                        const int32_t *gate_count, int gate_lo, int gate_hi)
{
    if (nq <= 0) return hipSuccess;
    const int total = P * k + (extra_lists ? k : 0);
    if (!only && !gate_count && sorted_lists && k <= 32 && total >= 1024 && P <= merge_max_sorted_lists(k)) {   // many short sorted lists
        const int Pt = P + (extra_lists ? 1 : 0);
        const size_t lds = merge_sorted_lds(Pt, k);
        const int lpl = (int)ceil_div(ceil_div(Pt, 4), 64);   // lists a lane owns
        static bool attr_set[4] = {false, false, false, false};   // per instantiation
        auto launch = [&](auto kern, int slot) -> hipError_t {
            if (!attr_set[slot]) {
                hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                   hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
                if (e != hipSuccess) return e;
                attr_set[slot] = true;
            }
            kern<<<(unsigned)nq, 256, lds, st>>>(lists, P, k, extra_lists, out_lists, seeds_out, ids, dists, qnorms, metric);
            return hipGetLastError();
        };
        if (lpl <= 1) return launch(merge_sorted_kernel<1>, 0);
        if (lpl <= 2) return launch(merge_sorted_kernel<2>, 1);
        if (lpl <= 4) return launch(merge_sorted_kernel<4>, 2);
        if (lpl <= 8) return launch(merge_sorted_kernel<8>, 3);
        return hipErrorInvalidValue;   // more than 2048 lists: merge_max_sorted_lists allows 1024
    }
    const int cap = next_pow2(total < 2 ? 2 : total);
    if (cap > 4096) return hipErrorInvalidValue;
    merge_kernel<<<(unsigned)nq, 256, (size_t)cap * sizeof(cand_t), st>>>(
        lists, P, k, extra_lists, cap, out_lists, seeds_out, ids, dists, qnorms, metric, only, gate_count, gate_lo, gate_hi);
    return hipGetLastError();
}

}  // namespace lpq
