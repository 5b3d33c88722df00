// Matrix-core search kernel, variant with the per-query lists of the k best in LDS (any k that
// fits, one 32-query block per wave for k > 16).  Same contraction, staging, epilogue and dump
// queue as search_mfma.hip; the drain inserts into LDS lists with a claim loop (one winner
// per query and round), which needs no registers per list entry.
#include "mfma_common.h"

namespace lpq {

namespace {

struct WaveState {   // pointers into the wave's private LDS region
    int *qvals;      // [16][QCAP]  accumulator r of dump s at qvals[r * QCAP + s]
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
    w.qrow = (int *)p;        p += QCAP * 4;
    w.qpar = (unsigned *)p;   p += QCAP * 4;
    w.qmeta = (int *)p;       p += QCAP * 4;
    w.thrE = (int *)p;        p += nqw * 4;
    w.cnt = (int *)p;         p += nqw * 4;
    w.worst = (int *)p;       p += nqw * 4;
    w.claim = (int *)p;       p += nqw * 4;
    w.lists = (cand_t *)p;    // 8-byte aligned: every size above is a multiple of 8
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
__device__ __noinline__ void drain_queue(unsigned char *wave_region, int nqw, int qcnt, int k, int64_t row_end, int lane)
{
    const WaveState w = carve_wave(wave_region, nqw);
    wave_lds_sync();
    for (int dbase = 0; dbase < qcnt; dbase += 64) {
        const int d = dbase + lane;
        const bool live = d < qcnt;
        const int meta = live ? w.qmeta[d] : 0;
        const int ql = meta & 255, hf = meta >> 8;
        const int rbase = live ? w.qrow[d] : 0;
        const unsigned pw = (L2 && live) ? w.qpar[d] : 0u;
        for (int r = 0; r < 16; ++r) {
            bool pend = false;
            cand_t c = 0;
            if (live) {
                const int e = w.qvals[r * QCAP + d];
                if (e >= w.thrE[ql]) {
                    const int off = 8 * (r >> 2) + 4 * hf + (r & 3);
                    const int64_t row = (int64_t)rbase + off;
                    const int b = (int)((pw >> off) & 1u);
                    c = make_cand(-(2 * e + b), (uint32_t)row);
                    pend = row < row_end && c < w.thrC[ql];
                }
            }
            while (__ballot(pend)) {  // one winner per query and round
                if (pend) w.claim[ql] = lane;
                wave_lds_sync();
                if (pend && w.claim[ql] == lane) {
                    if (c < w.thrC[ql]) list_insert(w, k, ql, c);
                    pend = false;
                }
                wave_lds_sync();
            }
        }
    }
}

template <int KS, int NB, bool L2>
__global__ __launch_bounds__(THREADS, 2) void search_mfma_lds_kernel(
    SearchArgs a, int64_t row0, int64_t row1, int S, int64_t split_rows, int qtiles,
    const cand_t *__restrict__ seeds, cand_t *__restrict__ lists_out)
{
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int NQW = 32 * NB;           // queries per wave
    constexpr int QT = WAVES * NQW;        // queries per workgroup
    constexpr int CPR = 2 * KS;            // 16-byte chunks per corpus row
    constexpr int SLOTS = CPR <= 2 ? 2 : (CPR <= 4 ? 4 : (CPR <= 8 ? 8 : 16));  // LDS slots per row
    constexpr int RS = KS <= 4 ? 64 : 32;  // corpus rows per stage
    constexpr int STAGE_BYTES = RS * SLOTS * 16;
    constexpr int IPW = RS * SLOTS / 64 / WAVES;   // async copy instructions per wave and stage
    constexpr int AUX_INTS = RS + 4;       // cinit[RS] then parity words
    static_assert(RS * SLOTS % (64 * WAVES) == 0 && IPW >= 1, "stage must split evenly over the waves");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform by construction
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

    unsigned char *ring = smem;
    int *aux = (int *)(smem + NSTG * STAGE_BYTES);
    unsigned char *wbase = (unsigned char *)(aux + NSTG * AUX_INTS);
    unsigned char *wregion = wbase + (size_t)wave * wave_region_bytes(NQW, k);
    const WaveState w = carve_wave(wregion, NQW);

    const int64_t q_first = (int64_t)qt * QT + wave * NQW;
    if (lane < NQW) {
        const int64_t gq = q_first + lane;
        const cand_t sd = (gq < a.nq) ? (seeds ? seeds[gq] : CAND_NONE) : 0;
        w.thrC[lane] = sd;
        w.thrE[lane] = thr_e(sd);
        w.cnt[lane] = 0;
        w.worst[lane] = 0;
    }
    wave_lds_sync();

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
    int a_off[KS];   // byte offset of this lane's A chunk of k-step ks inside a 32-row block of a stage
#pragma unroll
    for (int ks = 0; ks < KS; ++ks) a_off[ks] = col * (SLOTS * 16) + ((2 * ks + half) ^ swz<SLOTS>(col)) * 16;

    // ---- stage loader -----------------------------------------------------------------
    // Position p of a stage = LDS bytes [16p, 16p+16) = (row p / SLOTS, slot p % SLOTS).  Wave
    // `wave` copies positions [(wave*IPW + j)*64, +64) with instruction j; the lane's source
    // is the chunk that belongs in its slot, so every instruction reads whole rows.
    const unsigned ring_lds = lds_offset(ring), aux_lds = lds_offset(aux);
    const int lpt = IPW + ((L2 && wave < 2) ? 1 : 0);   // copies this wave issues per stage
    int src_off[IPW];   // byte offset of the lane's source chunk inside a stage of corpus rows
#pragma unroll
    for (int j = 0; j < IPW; ++j) {
        const int p = (wave * IPW + j) * 64 + lane;
        const int r = p / SLOTS, sl = p % SLOTS;
        int c = sl ^ swz<SLOTS>(r & 31);
        c = c < CPR ? c : CPR - 1;          // padding slots of non-power-of-two rows: any valid chunk
        src_off[j] = r * (32 * KS) + c * 16;
    }
#define LPQ_ISSUE(ST)                                                                                   \
    do {                                                                                                \
        const int st_ = (ST);                                                                           \
        const int64_t r0_ = rs + (int64_t)st_ * RS;                                                     \
        const int ring_slot_ = st_ % NSTG;                                                              \
        const int8_t *src_ = a.codes + r0_ * (32 * KS);                                                 \
        _Pragma("unroll") for (int j = 0; j < IPW; ++j)                                                 \
            async_copy16(src_ + src_off[j], ring_lds + ring_slot_ * STAGE_BYTES + (wave * IPW + j) * 1024); \
        if (L2 && wave == 0) {                                                                          \
            if (lane < RS) async_copy4(a.cinit + r0_ + lane, aux_lds + ring_slot_ * AUX_INTS * 4);      \
        } else if (L2 && wave == 1) {                                                                   \
            if (lane < RS / 32)                                                                         \
                async_copy4(a.parity + r0_ / 32 + lane, aux_lds + (ring_slot_ * AUX_INTS + RS) * 4);    \
        }                                                                                               \
    } while (0)

    const int T = (re > rs) ? (int)((re - rs + RS - 1) / RS) : 0;
    // Query fragments have landed before any copy is issued, so inside the loop only async
    // copies are ever outstanding on the vector-memory counter.
    __builtin_amdgcn_s_waitcnt(0x0F70);
    for (int st = 0; st < NSTG - 1 && st < T; ++st) LPQ_ISSUE(st);

    for (int t = 0; t < T; ++t) {
        // stages issued so far: 0 .. min(T-1, t+NSTG-2); wait until stage t has landed
        const int newer = (T - 1 < t + NSTG - 2 ? T - 1 : t + NSTG - 2) - t;
        wait_vmcnt(newer * lpt);
        __syncthreads();   // everybody's part of stage t is in LDS; stage t-1 is no longer read
        if (t + NSTG - 1 < T) LPQ_ISSUE(t + NSTG - 1);   // refills the slot of stage t-1

        const unsigned char *sb = ring + (size_t)(t % NSTG) * STAGE_BYTES;
        const int *cb = aux + (t % NSTG) * AUX_INTS;
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
                A[ks] = *reinterpret_cast<const v4i *>(sb + blk * 32 * (SLOTS * 16) + a_off[ks]);
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
                        drain_queue<L2>(wregion, NQW, qcnt, k, re, lane);
                        wave_lds_sync();
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
#pragma unroll
                            for (int r = 0; r < 16; ++r) w.qvals[r * QCAP + slot] = v[r];
                            w.qrow[slot] = rowbase;
                            w.qpar[slot] = L2 ? (unsigned)cb[RS + blk] : 0u;
                            w.qmeta[slot] = (nb * 32 + col) | (half << 8);
                        }
                        qcnt += __popcll(mask);
                    }
                }
            }
        }
    }
#undef LPQ_ISSUE

    drain_queue<L2>(wregion, NQW, qcnt, k, re, lane);
    wave_lds_sync();
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
    const int cpr = 2 * ks;
    const int slots = cpr <= 2 ? 2 : (cpr <= 4 ? 4 : (cpr <= 8 ? 8 : 16));
    const int rs = ks <= 4 ? 64 : 32;
    return (size_t)NSTG * rs * slots * 16 + (size_t)NSTG * (rs + 4) * 4 + WAVES * wave_region_bytes(32 * nb, k);
}

int nb_for(int k) { return k <= 16 ? 2 : 1; }

template <int KS, int NB, bool L2>
hipError_t launch_one(const SearchArgs &a, int64_t row0, int64_t row1, int S, const cand_t *seeds, cand_t *lists,
                      hipStream_t st)
{
    const int qt = 128 * NB;
    const int qtiles = (int)ceil_div(a.nq, qt);
    const int64_t split_rows = round_up(ceil_div(row1 - row0, S), 64);
    const size_t lds = lds_bytes(KS, NB, a.k);
    auto kern = search_mfma_lds_kernel<KS, NB, L2>;
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

bool mfma_lds_supported(int d_pad, int k)
{
    const int ks = d_pad / 32;
    if (d_pad % 32 || !(ks == 2 || ks == 3 || ks == 4 || ks == 6 || ks == 8)) return false;
    return k >= 1 && lds_bytes(ks, nb_for(k), k) <= 160 * 1024;
}

hipError_t launch_search_mfma_lds(const SearchArgs &a, int64_t row0, int64_t row1, int S, const cand_t *seeds,
                                  cand_t *lists, hipStream_t st)
{
    if (a.nq <= 0 || row1 <= row0) return hipSuccess;
    if (row0 % 64) return hipErrorInvalidValue;  // stages and parity words cover aligned blocks
    switch (a.d_pad / 32) {
    case 2: return launch_ks<2>(a, row0, row1, S, seeds, lists, st);
    case 3: return launch_ks<3>(a, row0, row1, S, seeds, lists, st);
    case 4: return launch_ks<4>(a, row0, row1, S, seeds, lists, st);
    case 6: return launch_ks<6>(a, row0, row1, S, seeds, lists, st);
    case 8: return launch_ks<8>(a, row0, row1, S, seeds, lists, st);
    default: return hipErrorInvalidValue;
    }
}

}  // namespace lpq
