// Matrix-core search kernel for gfx950: int8 query x corpus^T contraction on
// v_mfma_i32_32x32x32_i8 with the distance epilogue and the per-query top-k fused in.
//
// Work split.  A workgroup of 4 waves owns one query tile (4 x 32*NB queries) and one
// corpus split.  Each wave keeps the codes of its 32*NB queries in registers for the whole
// kernel (B operands); corpus rows stream through LDS in stages of 64 rows shared by the
// four waves (A operands), double buffered.  The corpus is the M side on purpose: the 16
// accumulators of a lane then belong to ONE query (column = lane % 32) and 16 different
// items, so the common-case epilogue is a max tree over the 16 values (v_max3) and one
// compare against that query's threshold: about 0.6 VALU operations per distance.
//
// Keys.  The accumulators start from cinit_j = -ceil(nx_j / 2) (0 for inner product), so
// the matrix core itself delivers E = dot - ceil(nx_j/2).  The exact ranking key is
// nx - 2 dot = -(2E + b) with b = nx & 1; the epilogue filters on E alone against a
// conservative threshold and the rare path restores b from one parity word per 32 items.
//
// Rare path.  A lane whose maximum passes dumps its 16 accumulators into a per-wave LDS
// queue (no atomics: the queue, the thresholds and the per-query lists are private to the
// wave).  When the queue is full the wave drains it densely - one (dump, accumulator) pair
// per lane - rebuilds exact candidates, inserts them into per-query lists of the k best
// (claim loop: one winner per query per round) and tightens the thresholds.
#include "lpq_internal.h"

namespace lpq {

namespace {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int WAVES = 4;
constexpr int THREADS = WAVES * 64;
constexpr int RS = 64;     // corpus rows per LDS stage
constexpr int QCAP = 64;   // dumps a wave can queue; one epilogue makes at most 64

__device__ inline void wave_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Largest E that cannot beat the candidate threshold c is one below the returned value:
// a candidate can only pass if E >= thr_e(c).
__device__ inline int thr_e(cand_t c)
{
    if (c == CAND_NONE) return INT32_MIN;
    if (c == 0) return INT32_MAX;  // a query slot that must never collect anything
    const long long t = (-(long long)cand_key(c)) >> 1;
    return t > INT32_MAX ? INT32_MAX : (t < INT32_MIN ? INT32_MIN : (int)t);
}

struct WaveState {   // pointers into the wave's private LDS region
    int *qvals;      // [QCAP][16]
    int *qrow;       // [QCAP] first row of the 32-row block the dump came from
    unsigned *qpar;  // [QCAP] parity word of that block
    int *qmeta;      // [QCAP] query slot | lane half << 8
    int *thrE;       // [NQW]
    cand_t *thrC;    // [NQW]
    int *cnt;        // [NQW]
    int *worst;      // [NQW]
    int *claim;      // [NQW]
    cand_t *lists;   // [NQW][k]
};

__host__ __device__ inline size_t wave_region_bytes(int nqw, int k)
{
    size_t b = (size_t)QCAP * 16 * 4 + (size_t)QCAP * 12;
    b += (size_t)nqw * (4 + 8 + 4 + 4 + 4);
    b += (size_t)nqw * k * 8;
    return (b + 15) & ~size_t(15);
}

__device__ inline WaveState carve_wave(unsigned char *p, int nqw)
{
    WaveState w;
    w.qvals = (int *)p;       p += QCAP * 16 * 4;
    w.thrC = (cand_t *)p;     p += nqw * 8;
    w.lists = nullptr;
    w.qrow = (int *)p;        p += QCAP * 4;
    w.qpar = (unsigned *)p;   p += QCAP * 4;
    w.qmeta = (int *)p;       p += QCAP * 4;
    w.thrE = (int *)p;        p += nqw * 4;
    w.cnt = (int *)p;         p += nqw * 4;
    w.worst = (int *)p;       p += nqw * 4;
    w.claim = (int *)p;       p += nqw * 4;
    p = (unsigned char *)(((uintptr_t)p + 7) & ~uintptr_t(7));
    w.lists = (cand_t *)p;
    return w;
}

// Put candidate c into the k-best list of query slot ql (called by one lane per query).
__device__ inline void list_insert(const WaveState &w, int k, int ql, cand_t c)
{
    cand_t *list = w.lists + (size_t)ql * k;
    int n = w.cnt[ql];
    if (n < k) {
        list[n] = c;
        w.cnt[ql] = ++n;
        if (n < k) return;
    } else {
        list[w.worst[ql]] = c;
    }
    cand_t mx = 0;
    int mp = 0;
    for (int i = 0; i < k; ++i) {
        const cand_t v = list[i];
        if (v > mx) { mx = v; mp = i; }
    }
    w.worst[ql] = mp;
    w.thrC[ql] = mx;
    w.thrE[ql] = thr_e(mx);
}

// Empty the wave's dump queue into its per-query lists.  Wave-uniform control flow.
template <bool L2>
__device__ inline void drain_queue(const WaveState &w, int qcnt, int k, int64_t row_end, int lane)
{
    wave_sync();
    const int total = qcnt * 16;
    for (int base = 0; base < total; base += 64) {
        const int idx = base + lane;
        bool pend = false;
        int ql = 0;
        cand_t c = 0;
        if (idx < total) {
            const int dump = idx >> 4, r = idx & 15;
            const int e = w.qvals[idx];
            const int meta = w.qmeta[dump];
            ql = meta & 255;
            if (e >= w.thrE[ql]) {
                const int off = 8 * (r >> 2) + 4 * (meta >> 8) + (r & 3);
                const int64_t row = (int64_t)w.qrow[dump] + off;
                const int b = L2 ? (int)((w.qpar[dump] >> off) & 1u) : 0;
                c = make_cand(-(2 * e + b), (uint32_t)row);
                pend = row < row_end && c < w.thrC[ql];
            }
        }
        while (__ballot(pend)) {  // one winner per query and round
            if (pend) w.claim[ql] = lane;
            wave_sync();
            if (pend && w.claim[ql] == lane) {
                if (c < w.thrC[ql]) list_insert(w, k, ql, c);
                pend = false;
            }
            wave_sync();
        }
    }
}

template <int KS, int NB, bool L2>
__global__ __launch_bounds__(THREADS, 2) void search_mfma_kernel(
    SearchArgs a, int64_t row0, int64_t row1, int S, int64_t split_rows, int qtiles,
    const cand_t *__restrict__ seeds, cand_t *__restrict__ lists_out)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int NQW = 32 * NB;           // queries per wave
    constexpr int QT = WAVES * NQW;        // queries per workgroup
    constexpr int STRIDE = 32 * KS + 16;   // LDS row stride: odd multiple of 16 bytes -> conflict-free b128 reads
    constexpr int CPR = 2 * KS;            // 16-byte chunks per row
    constexpr int CHUNKS = RS * CPR;
    constexpr int CH = (CHUNKS + THREADS - 1) / THREADS;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 31, half = lane >> 5;
    const int k = a.k;

    // XCD-aware work order: workgroups are dealt round-robin to the 8 XCDs, so give each XCD a
    // contiguous range of (split, query tile) pairs; neighbours on one XCD then stream the
    // same corpus split through that XCD's L2.
    const int total = qtiles * S;
    const int per = total / 8;
    const int b = blockIdx.x;
    const int wk = (b < per * 8) ? (b % 8) * per + b / 8 : b;
    const int s = wk / qtiles, qt = wk % qtiles;
    const int64_t rs = row0 + (int64_t)s * split_rows;
    const int64_t re = (rs + split_rows < row1) ? rs + split_rows : row1;

    unsigned char *stage = smem;
    int *cin = (int *)(smem + 2 * RS * STRIDE);
    unsigned *par = (unsigned *)(cin + 2 * RS);
    unsigned char *wbase = (unsigned char *)(par + 8);
    const WaveState w = carve_wave(wbase + (size_t)wave * wave_region_bytes(NQW, k), NQW);

    const int64_t q_first = (int64_t)qt * QT + wave * NQW;
    if (lane < NQW) {
        const int64_t gq = q_first + lane;
        const cand_t sd = (gq < a.nq) ? (seeds ? seeds[gq] : CAND_NONE) : 0;
        w.thrC[lane] = sd;
        w.thrE[lane] = thr_e(sd);
        w.cnt[lane] = 0;
        w.worst[lane] = 0;
    }
    wave_sync();

    v4i B[NB][KS];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            B[nb][ks] = *reinterpret_cast<const v4i *>(a.qcodes + (q_first + nb * 32 + col) * a.d_pad + ks * 32 + half * 16);
    int thr[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) thr[nb] = w.thrE[nb * 32 + col];
    int qcnt = 0;

    // Stage prefetch registers (named scalars, so they are never demoted to scratch memory).
    static_assert(CH >= 1 && CH <= 4, "stage loader handles up to 4 chunks per thread");
    uint4 pre0 = {0, 0, 0, 0}, pre1 = {0, 0, 0, 0}, pre2 = {0, 0, 0, 0}, pre3 = {0, 0, 0, 0};
    int pre_cin = 0;
    unsigned pre_par = 0;
#define LPQ_CHUNK_SRC(J) \
    reinterpret_cast<const uint4 *>(a.codes + (r0_ + ((tid + THREADS * (J)) % CHUNKS) / CPR) * a.d_pad + ((tid + THREADS * (J)) % CPR) * 16)
#define LPQ_CHUNK_DST(J) \
    reinterpret_cast<uint4 *>(stage + (size_t)buf_ * RS * STRIDE + ((tid + THREADS * (J)) / CPR) * STRIDE + ((tid + THREADS * (J)) % CPR) * 16)
#define LPQ_GLOAD(R0)                                                                         \
    do {                                                                                      \
        const int64_t r0_ = (R0);                                                             \
        if (CH > 0) pre0 = *LPQ_CHUNK_SRC(0);                                                 \
        if (CH > 1) pre1 = *LPQ_CHUNK_SRC(1);                                                 \
        if (CH > 2) pre2 = *LPQ_CHUNK_SRC(2);                                                 \
        if (CH > 3) pre3 = *LPQ_CHUNK_SRC(3);                                                 \
        if (L2 && tid < RS) pre_cin = a.cinit[r0_ + tid];                                     \
        if (L2 && tid >= 64 && tid < 64 + RS / 32) pre_par = a.parity[r0_ / 32 + (tid - 64)]; \
    } while (0)
#define LPQ_SSTORE(BUF)                                                                       \
    do {                                                                                      \
        const int buf_ = (BUF);                                                               \
        if (CH > 0 && tid + THREADS * 0 < CHUNKS) *LPQ_CHUNK_DST(0) = pre0;                   \
        if (CH > 1 && tid + THREADS * 1 < CHUNKS) *LPQ_CHUNK_DST(1) = pre1;                   \
        if (CH > 2 && tid + THREADS * 2 < CHUNKS) *LPQ_CHUNK_DST(2) = pre2;                   \
        if (CH > 3 && tid + THREADS * 3 < CHUNKS) *LPQ_CHUNK_DST(3) = pre3;                   \
        if (L2 && tid < RS) cin[buf_ * RS + tid] = pre_cin;                                   \
        if (L2 && tid >= 64 && tid < 64 + RS / 32) par[buf_ * 4 + (tid - 64)] = pre_par;      \
    } while (0)

    const int T = (re > rs) ? (int)((re - rs + RS - 1) / RS) : 0;
    if (T > 0) { LPQ_GLOAD(rs); LPQ_SSTORE(0); }
    // All loads so far (query fragments included) have landed: inside the loop only the stage
    // prefetch is ever outstanding, so the matrix instructions never wait on the memory counter.
    __builtin_amdgcn_s_waitcnt(0x0F70);  // vmcnt(0)
    __syncthreads();

    for (int t = 0; t < T; ++t) {
        if (t + 1 < T) LPQ_GLOAD(rs + (int64_t)(t + 1) * RS);
        const unsigned char *sb = stage + (size_t)(t & 1) * RS * STRIDE;
        const int *cb = cin + (t & 1) * RS;
#pragma unroll
        for (int blk = 0; blk < RS / 32; ++blk) {
            v16i c0;
            if (L2) {
#pragma unroll
                for (int g = 0; g < 4; ++g) {
                    const v4i v = *reinterpret_cast<const v4i *>(cb + blk * 32 + 8 * g + 4 * half);
                    c0[4 * g + 0] = v[0]; c0[4 * g + 1] = v[1]; c0[4 * g + 2] = v[2]; c0[4 * g + 3] = v[3];
                }
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) c0[i] = 0;
            }
            v4i A[KS];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
                A[ks] = *reinterpret_cast<const v4i *>(sb + (blk * 32 + col) * STRIDE + ks * 32 + half * 16);
            v16i acc[NB];
#pragma unroll
            for (int ks = 0; ks < KS; ++ks)
#pragma unroll
                for (int nb = 0; nb < NB; ++nb)
                    acc[nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[ks], B[nb][ks], ks == 0 ? c0 : acc[nb], 0, 0, 0);

            const int rowbase = (int)(rs + (int64_t)t * RS + blk * 32);
#pragma unroll
            for (int nb = 0; nb < NB; ++nb) {
                const v16i v = acc[nb];
                int m = max(max(v[0], v[1]), v[2]);
                m = max(max(m, v[3]), v[4]);
                m = max(max(m, v[5]), v[6]);
                m = max(max(m, v[7]), v[8]);
                m = max(max(m, v[9]), v[10]);
                m = max(max(m, v[11]), v[12]);
                m = max(max(m, v[13]), v[14]);
                m = max(m, v[15]);
                bool trip = m >= thr[nb];
                unsigned long long mask = __ballot(trip);
                if (mask) {
                    if (qcnt + __popcll(mask) > QCAP) {
                        drain_queue<L2>(w, qcnt, k, re, lane);
                        qcnt = 0;
#pragma unroll
                        for (int j = 0; j < NB; ++j) thr[j] = w.thrE[j * 32 + col];
                        trip = m >= thr[nb];
                        mask = __ballot(trip);
                    }
                    if (mask) {
                        const int below = __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),
                                                                    __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
                        if (trip) {
                            const int slot = qcnt + below;
                            v4i *dst = reinterpret_cast<v4i *>(w.qvals + slot * 16);
                            dst[0] = v4i{v[0], v[1], v[2], v[3]};
                            dst[1] = v4i{v[4], v[5], v[6], v[7]};
                            dst[2] = v4i{v[8], v[9], v[10], v[11]};
                            dst[3] = v4i{v[12], v[13], v[14], v[15]};
                            w.qrow[slot] = rowbase;
                            w.qpar[slot] = L2 ? par[(t & 1) * 4 + blk] : 0u;
                            w.qmeta[slot] = (nb * 32 + col) | (half << 8);
                        }
                        qcnt += __popcll(mask);
                    }
                }
            }
        }
        if (t + 1 < T) LPQ_SSTORE((t + 1) & 1);
        __syncthreads();
    }

#undef LPQ_GLOAD
#undef LPQ_SSTORE
#undef LPQ_CHUNK_SRC
#undef LPQ_CHUNK_DST

    drain_queue<L2>(w, qcnt, k, re, lane);
    wave_sync();
    if (lane < NQW) {
        const int64_t gq = q_first + lane;
        if (gq < a.nq) {
            cand_t *out = lists_out + ((size_t)gq * S + s) * k;
            const int n = w.cnt[lane];
            const cand_t *list = w.lists + (size_t)lane * k;
            for (int i = 0; i < k; ++i) out[i] = (i < n) ? list[i] : CAND_NONE;
        }
    }
}

size_t lds_bytes(int ks, int nb, int k)
{
    const size_t stride = 32 * ks + 16;
    return 2 * RS * stride + 2 * RS * 4 + 32 + WAVES * wave_region_bytes(32 * nb, k);
}

int nb_for(int k) { return k <= 16 ? 2 : 1; }

template <int KS, int NB, bool L2>
hipError_t launch_one(const SearchArgs &a, int64_t row0, int64_t row1, int S, const cand_t *seeds, cand_t *lists,
                      hipStream_t st)
{
    const int qt = 128 * NB;
    const int qtiles = (int)ceil_div(a.nq, qt);
    const int64_t split_rows = round_up(ceil_div(row1 - row0, S), RS);
    const size_t lds = lds_bytes(KS, NB, a.k);
    auto kern = search_mfma_kernel<KS, NB, L2>;
    static bool attr_set = false;  // per instantiation
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    kern<<<(unsigned)(qtiles * S), THREADS, lds, st>>>(a, row0, row1, S, split_rows, qtiles, seeds, lists);
    return hipGetLastError();
}

template <int KS>
hipError_t launch_ks(const SearchArgs &a, int64_t row0, int64_t row1, int S, const cand_t *seeds, cand_t *lists,
                     hipStream_t st)
{
    const bool l2 = a.metric == LPQ_METRIC_L2SQ;
    if (nb_for(a.k) == 2)
        return l2 ? launch_one<KS, 2, true>(a, row0, row1, S, seeds, lists, st)
                  : launch_one<KS, 2, false>(a, row0, row1, S, seeds, lists, st);
    return l2 ? launch_one<KS, 1, true>(a, row0, row1, S, seeds, lists, st)
              : launch_one<KS, 1, false>(a, row0, row1, S, seeds, lists, st);
}

}  // namespace

bool mfma_supported(int d_pad, int k)
{
    const int ks = d_pad / 32;
    if (d_pad % 32 || !(ks == 1 || ks == 2 || ks == 3 || ks == 4 || ks == 6 || ks == 8)) return false;
    return k >= 1 && lds_bytes(ks, nb_for(k), k) <= 160 * 1024;
}

size_t mfma_list_scratch_bytes(int64_t, int, int) { return 0; }

hipError_t launch_search_mfma(const SearchArgs &a, int64_t row0, int64_t row1, int S, const cand_t *seeds,
                              cand_t *lists, void *, hipStream_t st)
{
    if (a.nq <= 0 || row1 <= row0) return hipSuccess;
    if (row0 % 32) return hipErrorInvalidValue;  // parity words cover aligned 32-item blocks
    switch (a.d_pad / 32) {
    case 1: return launch_ks<1>(a, row0, row1, S, seeds, lists, st);
    case 2: return launch_ks<2>(a, row0, row1, S, seeds, lists, st);
    case 3: return launch_ks<3>(a, row0, row1, S, seeds, lists, st);
    case 4: return launch_ks<4>(a, row0, row1, S, seeds, lists, st);
    case 6: return launch_ks<6>(a, row0, row1, S, seeds, lists, st);
    case 8: return launch_ks<8>(a, row0, row1, S, seeds, lists, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace lpq
