// Matrix-core search kernel for gfx950: int8 query x corpus^T contraction on
// v_mfma_i32_32x32x32_i8 with the distance epilogue and the per-query top-k fused in.
//
// Work split.  A workgroup of 4 waves owns one query tile (256 queries, 64 per wave) and one
// corpus split.  Each wave keeps the codes of its 64 queries in registers for the whole
// kernel (B operands); corpus rows stream through an LDS ring of NST stages shared by the
// four waves (A operands): two stages of 128 rows for rows of up to 128 bytes, two or four of
// 64 rows otherwise.  The ring is filled by asynchronous global->LDS loads
// (global_load_lds_dwordx4) issued NST-1 stages ahead, one workgroup barrier per stage; rows sit
// in LDS row-major with an XOR swizzle of their 16-byte chunks, which keeps the global side fully
// coalesced and the ds_read_b128 of the A operands free of bank conflicts.  Inside a 32-row block
// each block of 32 queries gets its matrix instructions as one chain, and the filter epilogue of
// a block runs one chain later (the last one after the first chain of the next row block), so the
// epilogue issues while the matrix core is busy.
//
// The corpus is the M side on purpose: the 16 accumulators of a lane then belong to ONE
// query (column = lane % 32) and 16 different items, so the common-case epilogue is a max
// tree over the 16 values (v_max3) and one compare against that query's threshold: about
// 0.6 VALU operations per distance.
//
// Keys.  The accumulators start from cinit_j = -ceil(nx_j / 2) (0 for inner product), so
// the matrix core itself delivers E = dot - ceil(nx_j/2).  The exact ranking key is
// nx - 2 dot = -(2E + b) with b = nx & 1; the epilogue filters on E alone against a
// conservative threshold and the rare path restores b from one parity word per 32 items.
//
// Rare path.  A lane whose maximum passes dumps its 16 accumulators into a per-wave LDS
// queue (no atomics: the queue and the thresholds are private to the wave).  Queues are
// drained by all four waves together at a stage boundary as soon as one of them is half
// full (a wave that overflows in between drains alone).  A drain scans the dumps densely,
// compacts the exact candidates that still beat their query's threshold, and hands them to
// the lane that owns the query (lane q of the wave owns query q): the owner keeps the k best
// in registers as a sorted list and inserts with one compare-exchange pass.
//
// Collecting mode (KCAP = 0, for k beyond what fits in registers).  The threshold of a query stays
// at its seed for the whole scan and a drain appends every exact candidate that beats it to a
// region of global memory owned by this (query, split[, wave]): no lists, no atomics outside the
// wave's LDS counters.  The seed threshold is reached by at least k items, so the k best are among
// the collected ones; a later kernel selects them (or flags a query whose region overflowed for an
// exact redo: by the generic kernel, or, when many are flagged, by a launch of this kernel in list
// mode that skips query tiles without a flagged query).  With short rows and many queries a wave
// holds 128 queries (NB = 4 blocks of 32) instead of 64.
//
// Row-split launches (RSPLIT, at most 64 queries).  The four waves (two on rows of more than 128
// bytes) share the 64 queries and split the rows of a stage, 32 rows per wave; each wave copies,
// waits for and reads only its own 32 rows, so there is no workgroup barrier and the launch runs at
// the speed the corpus streams in.  PACK: the rows hold two 4-bit codes per byte and are spread over
// the operand registers after the LDS read (row-split launches, and the collecting scan and seeding
// pass of large batches).
//
// Seeding pass (SEED = true).  The same pipeline with collection switched off: every lane
// only tracks the maximum E it has seen per segment of its split.  Each (segment, lane half)
// is a group of items disjoint from the others, so the k-th largest group maximum of a query
// is a value that at least k items reach: an upper bound on the k-th best key that costs
// nothing but the contraction itself.  The main pass starts from it.  The pass reads a systematic
// sample of the corpus: whole stages at a stride, or runs of 8 rows gathered from places far
// apart, so that rows stored next to each other fall into different groups.
#include <type_traits>

#include "mfma_common.h"
#include "wave_ops.h"

namespace lpq {

namespace {

// Timing ablations (results then meaningless) exist only in builds compiled with -DLPQ_ABLATION;
// in the shipped library the value is the constant 0 and the branches on it vanish.
#ifdef LPQ_ABLATION
#define LPQ_DRY(a) ((a).dry_run)
#else
#define LPQ_DRY(a) 0
#endif

// After the thresholds have been re-read from LDS on a rare path: wait for them there, as an
// instruction the compiler's wait-count bookkeeping sees.  Otherwise the registers count as "load
// pending" where the rare path rejoins the common one, and every later threshold compare of the
// common path gets a "wait for all LDS loads" in front of it, also right after the operand loads of
// the next row block were issued.  (Measured: the same time either way on the benchmark workload -
// those loads have returned by then; kept so that the common path only waits where it consumes.)
#define LPQ_LGKM_SETTLED() __builtin_amdgcn_s_waitcnt(0xC07F)   /* lgkmcnt(0); vmcnt, expcnt untouched */

// Instruction order of one chain and the filter epilogue of the chain before it (one scheduling
// region: it ends at the epilogue's branch): two matrix instructions first, then the max tree in the
// shadow of the second one, then the remaining matrix instructions with the rest of the vector work
// between them; without it the compiler puts seven of the nine vector instructions and the idle
// cycles their operands need behind the first matrix instruction.  Measured on one box (main scan of
// the benchmark workload): 0.934 -> 0.917 ms; 1.2M x 100, inner product: 1.101 -> 1.079 ms.
#define LPQ_SCHED_CHAIN()                                                                               \
    do {                                                                                                \
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);   /* 2 matrix instructions */                \
        __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);   /* 5 vector instructions */                \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                              \
        __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);                                              \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                              \
    } while (0)

constexpr int NQW = 64;      // queries per wave in list mode = lanes per wave: lane q owns query q
constexpr int TRIG = 32;     // queue fill that asks for a joint drain at the next stage boundary
constexpr int SVCAP = 128;   // compacted candidates buffered before they are handed to owners

struct MfmaIo {     // what a launch reads and writes besides the corpus and the queries
    const cand_t *seeds;   // [nq] starting thresholds, or null
    cand_t *lists;         // list mode: [nq][S][k]
    int32_t *gmax;         // seeding pass: [nq_pad][G] group maxima
    int SEG;               // seeding pass: segments per split
    cand_t *cbuf;          // collecting mode: [nq][SS][Cs] regions, SS = S (x waves when rows are split)
    int32_t *ccnt;         // collecting mode: [nq][SS] candidates offered to each region (may exceed Cs)
    int Cs;
    int64_t split_stride;       // first row of split s is row0 + s * split_stride; 0: splits follow each other
    int64_t split_stride_rows;  // with a stride: rows per split
    int64_t stage_stride;       // seeding pass: first rows of consecutive stages are this far apart (0: adjacent)
    // Seeding pass over a finer systematic sample (not for row-split launches): piece P = rows
    // [P * piece_stride, + 8); split s takes pieces s, s + S, s + 2S, ..., eight to a stage,
    // piece_stages stages.  0: stages of 64 consecutive rows as above.
    int64_t piece_stride;
    int piece_stages;
};

struct WaveQ {      // pointers into the wave's private LDS region
    cand_t *thrC;   // [NQW] exact threshold candidate per query
    cand_t *svc;    // [SVCAP] compacted candidates
    int *qvals;     // [QCAP][16] the 16 accumulators of dump s at qvals[16 s ..]
    v4i *qmeta;     // [QCAP] (first row of the dump's 32-row block, its parity word, query slot | lane half << 8, -)
    int *thrE;      // [NQW] conservative threshold on E
    int *mbox;      // [NQW] lane whose candidate the owner takes this round, or -1 (collecting mode: region fill)
    int *svq;       // [SVCAP] query slot of each compacted candidate
};

// bytes of a wave's region, for qw queries per wave (LDS is what limits two workgroups per CU)
constexpr size_t waveq_bytes(int qw) { return (size_t)qw * 8 + SVCAP * 8 + QCAP * 16 * 4 + QCAP * 16 + (size_t)qw * 8 + SVCAP * 4; }

__device__ __forceinline__ WaveQ carve_waveq(unsigned char *p, int qw)
{
    WaveQ w;
    w.thrC = (cand_t *)p;    p += qw * 8;
    w.svc = (cand_t *)p;     p += SVCAP * 8;
    w.qvals = (int *)p;      p += QCAP * 16 * 4;
    w.qmeta = (v4i *)p;      p += QCAP * 16;
    w.thrE = (int *)p;       p += qw * 4;
    w.mbox = (int *)p;       p += qw * 4;
    w.svq = (int *)p;
    return w;
}

__device__ __forceinline__ cand_t shfl_cand(cand_t c, int src_lane)
{
    const unsigned lo = (unsigned)__shfl((int)(unsigned)c, src_lane, 64);
    const unsigned hi = (unsigned)__shfl((int)(unsigned)(c >> 32), src_lane, 64);
    return ((cand_t)hi << 32) | lo;
}

// Sorted (ascending) list of the KCAP best candidates of one query, in registers.
template <int KCAP>
__device__ __forceinline__ void reglist_insert(cand_t (&lst)[KCAP], cand_t c, bool doit)
{
#pragma unroll
    for (int i = 0; i < KCAP; ++i) {
        const cand_t t = lst[i];
        const bool lt = doit && c < t;
        lst[i] = lt ? c : t;
        c = lt ? t : c;
    }
}

// Hand the first `svcnt` compacted candidates to the owner lanes, then publish the owners'
// new thresholds.  Wave-uniform control flow; lane q owns query q.
template <int KCAP>
__device__ __forceinline__ void give_to_owners(const WaveQ &w, int svcnt, int lane, cand_t (&lst)[KCAP], cand_t seedC)
{
    wave_lds_sync();
    for (int base = 0; base < svcnt; base += 64) {
        const int idx = base + lane;
        bool pend = idx < svcnt;
        const cand_t c = pend ? w.svc[idx] : 0;
        const int ql = pend ? w.svq[idx] : 0;
        while (__ballot(pend)) {   // every round each query with candidates left takes one
            if (pend) w.mbox[ql] = lane;
            wave_lds_sync();
            const int wl = w.mbox[lane];             // owner: the lane whose candidate I take, or -1
            if (wl >= 0) w.mbox[lane] = -1;
            const cand_t cw = shfl_cand(c, wl & 63);
            const int taken = __shfl(wl, ql, 64);    // sender: which lane my query's owner took
            reglist_insert<KCAP>(lst, cw, wl >= 0);
            if (pend && taken == lane) pend = false;
            wave_lds_sync();
        }
    }
    const cand_t kth = lst[KCAP - 1];
    const cand_t tc = kth < seedC ? kth : seedC;
    w.thrC[lane] = tc;
    w.thrE[lane] = thr_e(tc);
    wave_lds_sync();
}

// Collecting mode: append the first `svcnt` compacted candidates to their queries' regions.
// The stores stay in flight; they only make the counted waits for the ring more conservative.
__device__ __forceinline__ void append_collected(const WaveQ &w, int svcnt, int lane, cand_t *cbase, size_t qstride,
                                                 int Cs)
{
    wave_lds_sync();
    for (int base = 0; base < svcnt; base += 64) {
        const int idx = base + lane;
        if (idx < svcnt) {
            const cand_t c = w.svc[idx];
            const int ql = w.svq[idx];
            const int pos = atomicAdd(&w.mbox[ql], 1);
            if (pos < Cs) cbase[(size_t)ql * qstride + pos] = c;
        }
    }
    wave_lds_sync();
}

// Empty the wave's dump queue.  Wave-uniform control flow.
template <bool L2, int KCAP, int LK>
__device__ __forceinline__ void drain_queue(const WaveQ &w, int qcnt, int64_t row_end, int lane,
                                            cand_t (&lst)[LK], cand_t seedC, cand_t *cbase, size_t qstride, int Cs)
{
    if (qcnt <= 0) return;
    wave_lds_sync();
    // Lanes cover (dump, accumulator) pairs: DW = pow2 >= qcnt dumps side by side, 64/DW
    // accumulator indices per step.
    int lg = 32 - __builtin_clz((unsigned)(qcnt > 1 ? qcnt - 1 : 1) | 1u);
    if (qcnt <= 1) lg = 0;
    if (lg > 6) lg = 6;
    const int d = lane & ((1 << lg) - 1), rsub = lane >> lg, rstep = 64 >> lg;
    const bool live = d < qcnt;
    v4i m4 = {0, 0, 0, 0};
    if (live) m4 = w.qmeta[d];
    const int meta = m4[2];
    const int ql = meta & 255, hf = meta >> 8;
    const int rbase = m4[0];
    const unsigned pw = L2 ? (unsigned)m4[1] : 0u;
    // A lane walks the accumulators of its dump starting from a dump-dependent index, so that the
    // lanes of one step (dumps 64 bytes apart) fall on different banks.
    const int rot = (d >> 2) * rstep;
    int svcnt = 0;
    for (int r0 = 0; r0 < 16; r0 += rstep) {
        const int r = (r0 + rsub + rot) & 15;
        bool pass = live && rsub < 16;
        cand_t c = 0;
        if (pass) {
            const int e = w.qvals[d * 16 + r];
            pass = e >= w.thrE[ql];
            if (pass) {
                const int off = 8 * (r >> 2) + 4 * hf + (r & 3);
                const int64_t row = (int64_t)rbase + off;
                const int b = (int)((pw >> off) & 1u);
                c = make_cand(-(2 * e + b), (uint32_t)row);
                pass = row < row_end && c < w.thrC[ql];
            }
        }
        const unsigned long long mask = __ballot(pass);
        if (mask) {
            const int pos = svcnt + __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),
                                                               __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u));
            if (pass) { w.svc[pos] = c; w.svq[pos] = ql; }
            svcnt += __popcll(mask);
            if (svcnt > SVCAP - 64) {
                if constexpr (KCAP > 0) give_to_owners<KCAP>(w, svcnt, lane, lst, seedC);
                else append_collected(w, svcnt, lane, cbase, qstride, Cs);
                svcnt = 0;
            }
        }
    }
    if (svcnt) {
        if constexpr (KCAP > 0) give_to_owners<KCAP>(w, svcnt, lane, lst, seedC);
        else append_collected(w, svcnt, lane, cbase, qstride, Cs);
    }
}

constexpr bool big_stage(int kcap, bool seed, bool rsplit, int nb, bool pack, int ks = 4) { return !seed && !rsplit && !pack && ks <= 4; }
constexpr int ring_depth(int ks, bool rsplit, bool pack, bool big = false) { return big ? 2 : (rsplit ? (pack ? 4 : 3) : (ks <= 4 ? 4 : 2)); }

template <int KS, bool L2, int KCAP, bool SEED, int NW, bool RSPLIT, int NB, bool PACK>
__global__ __launch_bounds__(NW * 64, 2) void search_mfma_kernel(
    SearchArgs a, int64_t row0, int64_t row1, int S, int64_t split_rows, int qtiles, MfmaIo o)
{
    extern __shared__ __align__(16) unsigned char smem[];
    // NB blocks of 32 queries per wave: 2, or 4 (128 queries per wave, 512 per workgroup) in the
    // collecting mode of large batches and its seeding pass, where no lane owns a list.
    static_assert(NB == 2 || (NB == 4 && (KCAP == 0 || SEED) && !RSPLIT), "four query blocks: no register lists");
    constexpr int QW = NB * 32;            // queries per wave
    constexpr bool COLLECT = !SEED && KCAP == 0;
    constexpr int LK = KCAP > 0 ? KCAP : 1;
    const cand_t *__restrict__ seeds = o.seeds;
    cand_t *__restrict__ lists_out = o.lists;
    int32_t *__restrict__ gmax = o.gmax;
    const int SEG = o.SEG;
    // RSPLIT (few queries): the waves of a workgroup share ONE 64-query tile and split the rows of
    // a stage between them (one 32-row block each), so no matrix work is spent on padding queries.
    // Every wave then copies, waits for and reads only its own quarter of each stage: the waves run
    // without any workgroup barrier and the path is bound by how fast the corpus streams in.
    constexpr int QT = RSPLIT ? QW : NW * QW;   // queries per workgroup
    // PACK: the corpus holds two 4-bit codes per byte, stored as u = code + 8 (0..15): rows are half
    // as long in HBM and in LDS; a lane reads 8 bytes per k-step and spreads the nibbles over its
    // four operand registers (low nibbles of a dword, then its high nibbles), which permutes the
    // 16 codes of the lane inside the k-step; the caller hands in query codes permuted the same
    // way.  The matrix core then delivers dot(u, q) = dot(code, q) + 8 sum(q): a constant per query,
    // which shifts every key of a query alike and is taken out when the result is written.
    static_assert(!PACK || RSPLIT || ((KCAP == 0 || SEED) && KS >= 3),
                  "packed rows: row-split launches, or the collecting scan and its seeding pass on rows of 48 bytes or more");
    constexpr int CPR = PACK ? KS : 2 * KS;   // 16-byte chunks per corpus row
    constexpr int ROWB = 16 * CPR;            // bytes per corpus row
    constexpr int SLOTS = CPR <= 2 ? 2 : (CPR <= 4 ? 4 : (CPR <= 8 ? 8 : 16));  // LDS slots per row
    // Scans of rows of up to 128 bytes whose waves share a stage (all but the row-split launches,
    // the seeding pass and packed rows) take stages of 128 rows through a two-deep ring (the same
    // 32 KB of LDS as four stages of 64): half as many workgroup barriers and copy waits per row.
    // Measured on the benchmark workload: 1.283 -> 1.171 ms per 10 000 queries (k = 100: 2.06 ->
    // 1.82; 10M x 96: 10.0 -> 8.7 ms; 256 queries on 10M x 96: 0.394 -> 0.333 ms).  Longer rows
    // would need 64 KB for such a ring, which no longer fits two workgroups per CU.
    constexpr bool BIG = big_stage(KCAP, SEED, RSPLIT, NB, PACK, KS);
    constexpr int RS = RSPLIT ? 32 * NW : (BIG ? 128 : 64);   // corpus rows per stage
    // LDS ring depth.  Row-split launches: 3, or 4 for the half-size packed stages (2.5 % faster);
    // rings of 6 and 8 packed stages measured 55 % slower, as deeper rings did for unpacked rows.
    // Shared stages: 2 for the 128-row stages and for rows of more than 128 bytes (3 measured 36 %
    // and 1.8 % slower there), 4 for the 64-row stages of the seeding pass on short rows, whose
    // stages are gathered from far apart and need the lead (3: 1.5 % slower, 2: 4 %).
    constexpr int NST = ring_depth(KS, RSPLIT, PACK, BIG);
    static_assert(!RSPLIT || ROWB <= 128 || (NW == 2 && (KCAP == 0 || SEED)),
                  "row-split staging: four waves on rows of up to 128 bytes, two on longer ones (no register lists there)");
    constexpr int STAGE_BYTES = RS * SLOTS * 16;
    constexpr int IPW = RS * SLOTS / 64 / NW;   // async copy instructions per wave and stage
    constexpr int AUX_INTS = RS + 4;       // cinit[RS] then parity words
    static_assert(RS * SLOTS % (64 * NW) == 0 && IPW >= 1, "stage must split evenly over the waves");
    static_assert((NST - 1) * (IPW + (RSPLIT ? 2 : 1)) <= 63, "wait_vmcnt covers 0..63");
    static_assert(!RSPLIT || IPW * 64 == 32 * SLOTS, "row-split: a wave copies exactly its own 32 rows");

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
    const int wk = (a.work_order != 3 && b < per * 8) ? (b % 8) * per + b / 8 : b;
    const int s = (a.work_order == 2) ? wk % S : wk / qtiles;
    const int qt = (a.work_order == 2) ? wk / S : wk % qtiles;
    // Stage st of this split starts at row rs + st * sstride.  Splits are contiguous row ranges with
    // adjacent stages, except: a collecting scan deals the stages of the corpus round-robin to its
    // splits (ILV), so that the candidates of a query spread evenly over the splits' regions however
    // the corpus is ordered, and so does every row-split scan (workgroups that advance together then
    // read one moving window of the corpus, which measured 5-10 % faster than 256-512 separate
    // streams); and the seeding pass may sample one stage every stage_stride rows.
    constexpr bool ILV = !SEED && (KCAP == 0 || RSPLIT);
    constexpr int RS_ = RS;
    const int64_t rs = ILV ? row0 + (int64_t)s * RS_ : row0 + (int64_t)s * o.split_stride;
    const int64_t re = ILV ? row1 : ((rs + split_rows < row1) ? rs + split_rows : row1);
    const int64_t sstride = ILV ? (int64_t)S * RS_ : ((SEED && o.stage_stride) ? o.stage_stride : RS_);

    unsigned char *ring = smem;
    int *aux = (int *)(smem + NST * STAGE_BYTES);
    int *flags = aux + NST * AUX_INTS;           // [2][8] joint-drain requests, double buffered
    const WaveQ w = carve_waveq((unsigned char *)(flags + 16) + (size_t)wave * waveq_bytes(NB * 32), NB * 32);

    const int64_t q_first = (int64_t)qt * QT + (RSPLIT ? 0 : wave * QW);

    if constexpr (!SEED && !RSPLIT) {
        if (a.redo_flags) {   // redo pass: only if the flagged queries are many, and only tiles that hold one
            if (*a.redo_count <= a.redo_min) return;   // the same answer in every thread of the grid
            const int64_t t0 = (int64_t)qt * QT;
            int mine = 0;
            for (int64_t qq = t0 + tid; qq < t0 + QT && qq < a.nq; qq += NW * 64) mine |= a.redo_flags[qq];
            // workgroup-wide OR through the (still unused) first word of the ring: the kernel has no
            // static LDS, which the 160 KB dynamic limit set at launch leaves no room for
            int *vote = reinterpret_cast<int *>(ring);
            if (tid == 0) *vote = 0;
            __syncthreads();
            if (mine) atomicOr(vote, 1);
            __syncthreads();
            const int any = *vote;
            __syncthreads();   // everyone has read the vote before the ring is filled
            if (!any) return;  // the same answer in every thread of the workgroup
        }
    }
    if constexpr (!SEED && RSPLIT) {   // row-split launches hold one tile of queries: the count alone decides
        if (a.redo_flags && *a.redo_count <= a.redo_min) return;
    }

    // ---- owner state (lane q owns query q of this wave) ------------------------------
    cand_t lst[LK];
    cand_t seedC = 0;
    // collecting mode: this wave's regions are cbase + query slot * qstride
    const int SS = S * (RSPLIT ? NW : 1), sub = s * (RSPLIT ? NW : 1) + (RSPLIT ? wave : 0);
    cand_t *cbase = COLLECT ? o.cbuf + ((size_t)q_first * SS + sub) * o.Cs : nullptr;
    const size_t qstride = (size_t)SS * o.Cs;
    if (!SEED) {
        const int64_t gq = q_first + lane;
        seedC = (gq < a.nq && (LPQ_DRY(a) == 0 || LPQ_DRY(a) >= 5)) ? (seeds ? seeds[gq] : CAND_NONE) : 0;
        // slots beyond k are pinned to the smallest candidate, so lst[KCAP-1] is the k-th best
#pragma unroll
        for (int i = 0; i < LK; ++i) lst[i] = (i < KCAP - k) ? 0 : CAND_NONE;
        w.thrC[lane] = seedC;
        w.thrE[lane] = thr_e(seedC);
        w.mbox[lane] = COLLECT ? 0 : -1;
        if constexpr (QW > 64) {   // the second 64 queries of the wave
            const int64_t gq2 = gq + 64;
            const cand_t s2 = (gq2 < a.nq && (LPQ_DRY(a) == 0 || LPQ_DRY(a) >= 5)) ? (seeds ? seeds[gq2] : CAND_NONE) : 0;
            w.thrC[64 + lane] = s2;
            w.thrE[64 + lane] = thr_e(s2);
            w.mbox[64 + lane] = 0;
        }
    }
    wave_lds_sync();

    v4i B[NB][KS];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            B[nb][ks] = *reinterpret_cast<const v4i *>(a.qcodes + (q_first + nb * 32 + col) * a.d_pad + ks * 32 + half * 16);
    // Seeding pass: running maxima per group of rows, GR groups per lane.  GR = 16 (one group per
    // accumulator, so that neighbouring rows fall into different groups) gives tighter bounds on a
    // corpus stored in sorted order but measured 50 % slower overall on the benchmark workload (the
    // extra registers spill in the 128-queries-per-wave kernel), so one group per lane half it is.
    constexpr int GR = 1;
    int thr[NB], gm[NB][GR];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        thr[nb] = SEED ? INT32_MAX : w.thrE[nb * 32 + col];
#pragma unroll
        for (int r = 0; r < GR; ++r) gm[nb][r] = INT32_MIN;
    }
    int qcnt = 0;
    int a_off[KS];   // byte offset of this lane's A chunk of k-step ks inside a 32-row block of a stage
#pragma unroll
    for (int ks = 0; ks < KS; ++ks)
        a_off[ks] = PACK ? col * (SLOTS * 16) + (ks ^ swz<SLOTS>(col)) * 16 + half * 8
                         : col * (SLOTS * 16) + ((2 * ks + half) ^ swz<SLOTS>(col)) * 16;

    // ---- stage loader -----------------------------------------------------------------
    // Position p of a stage = LDS bytes [16p, 16p+16) = (row p / SLOTS, slot p % SLOTS).  Wave
    // `wave` copies positions [(wave*IPW + j)*64, +64) with instruction j; the lane's source
    // is the chunk that belongs in its slot, so every instruction reads whole rows.
    const unsigned ring_lds = lds_offset(ring), aux_lds = lds_offset(aux);
    const int lpt = IPW + (!L2 ? 0 : (RSPLIT ? 2 : (wave < RS / 64 + 1 ? 1 : 0)));   // copies this wave issues per stage
    // Seeding pass by pieces: the 64 rows of a stage are eight runs of 8 rows taken S * piece_stride
    // rows apart, so that neighbouring rows of the corpus fall into different splits (and groups).
    constexpr bool CAN_PIECES = SEED && !RSPLIT;
    const bool pieces = CAN_PIECES && o.piece_stride > 0;
    const int64_t piece_gap = pieces ? (int64_t)S * o.piece_stride : 0;   // rows between the pieces of a stage
    int src_off[IPW];   // byte offset of the lane's source chunk relative to the first row of a stage (of its piece)
#pragma unroll
    for (int j = 0; j < IPW; ++j) {
        const int p = (wave * IPW + j) * 64 + lane;
        const int r = p / SLOTS, sl = p % SLOTS;
        int c = sl ^ swz<SLOTS>(r & 31);
        c = c < CPR ? c : CPR - 1;          // padding slots of non-power-of-two rows: any valid chunk
        src_off[j] = (pieces ? (r & 7) : r) * ROWB + c * 16;
    }
    // Row of the accumulator seed that wave 0's lane brings (non-row-split launches).  It is worked
    // out from the lane number where it is used, behind a barrier for the optimiser: kept in a
    // register across the loop, the seeding pass of 128 queries per wave spills it, and a reload
    // from scratch waits for every copy in flight (they share the vector-memory counter).
    // (Only that kernel: where nothing spills, carrying the addresses measured 1 to 4 % faster.)
    constexpr bool REFORM = CAN_PIECES && NB == 4 && KS == 4;
#define LPQ_OPAQUE(X) asm volatile("" : "+v"(X))
#define LPQ_ISSUE(ST)                                                                                   \
    do {                                                                                                \
        const int st_ = (ST);                                                                           \
        int lane_ = lane;                                                                               \
        if (REFORM) LPQ_OPAQUE(lane_);                                                                  \
        const int64_t cin_off = pieces ? (int64_t)(lane_ >> 3) * piece_gap + (lane_ & 7) : (int64_t)wave * 64 + lane_; \
        const int64_t r0_ = pieces ? ((int64_t)s + (int64_t)S * 8 * st_) * o.piece_stride                \
                                   : rs + (int64_t)(LPQ_DRY(a) == 7 ? (st_ & 1) : st_) * sstride;       \
        const int ring_slot_ = st_ % NST;                                                               \
        const int8_t *src_ = a.codes + r0_ * ROWB;                                                      \
        _Pragma("unroll") for (int j = 0; j < IPW; ++j) {                                               \
            /* pieces: the lane's row belongs to piece (row of the stage) / 8, which is the same for */ \
            /* all lanes of the instruction when a row takes 8 slots or more                          */ \
            const int piece_ = SLOTS >= 8 ? (((wave * IPW + j) * 64) / SLOTS) >> 3                      \
                                          : (((wave * IPW + j) * 64 + lane_) / SLOTS) >> 3;             \
            const int64_t far_ = pieces ? (int64_t)piece_ * piece_gap * ROWB : 0;                       \
            int near_ = src_off[j];   /* stays one register: the 64-bit sum is formed here */           \
            if (REFORM) LPQ_OPAQUE(near_);                                                              \
            async_copy16(src_ + far_ + near_, ring_lds + ring_slot_ * STAGE_BYTES + (wave * IPW + j) * 1024); \
        }                                                                                               \
        if (L2 && RSPLIT) { /* each wave brings the seeds and the parity word of its own block */       \
            if (lane < 32)                                                                              \
                async_copy4(a.cinit + r0_ + wave * 32 + lane, aux_lds + (ring_slot_ * AUX_INTS + wave * 32) * 4); \
            if (lane < 1)                                                                               \
                async_copy4(a.parity + r0_ / 32 + wave, aux_lds + (ring_slot_ * AUX_INTS + RS + wave) * 4); \
        } else if (L2 && wave < RS / 64) {                                                              \
            async_copy4(a.cinit + r0_ + cin_off, aux_lds + (ring_slot_ * AUX_INTS + wave * 64) * 4);     \
        } else if (L2 && wave == RS / 64) {                                                             \
            if (lane < RS / 32)                                                                         \
                async_copy4(a.parity + r0_ / 32 + lane, aux_lds + (ring_slot_ * AUX_INTS + RS) * 4);    \
        }                                                                                               \
    } while (0)

    // Operands of one 32-row block, LDS -> registers: the A fragments, the accumulator seeds
    // of this lane's 16 rows, and the block's parity word.
#define LPQ_LOAD_BLOCK(TT, BLK, AREG, CREG, PREG)                                                       \
    do {                                                                                                \
        const unsigned char *sb_ = ring + (size_t)((TT) % NST) * STAGE_BYTES + (BLK) * 32 * (SLOTS * 16); \
        const int *cb_ = aux + ((TT) % NST) * AUX_INTS;                                                 \
        _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                             \
            if (PACK) {                                                                                 \
                const v2i w_ = *reinterpret_cast<const v2i *>(sb_ + a_off[ks]);                         \
                AREG[ks] = v4i{w_[0] & 0x0F0F0F0F, (int)(((unsigned)w_[0] >> 4) & 0x0F0F0F0Fu),         \
                               w_[1] & 0x0F0F0F0F, (int)(((unsigned)w_[1] >> 4) & 0x0F0F0F0Fu)};        \
            } else {                                                                                    \
                AREG[ks] = *reinterpret_cast<const v4i *>(sb_ + a_off[ks]);                             \
            }                                                                                           \
        }                                                                                               \
        if (L2) {                                                                                       \
            _Pragma("unroll") for (int g = 0; g < 4; ++g) {                                             \
                const v4i v_ = *reinterpret_cast<const v4i *>(cb_ + (BLK) * 32 + 8 * g + 4 * half);     \
                CREG[4 * g + 0] = v_[0]; CREG[4 * g + 1] = v_[1];                                       \
                CREG[4 * g + 2] = v_[2]; CREG[4 * g + 3] = v_[3];                                       \
            }                                                                                           \
            PREG = (unsigned)cb_[RS + (BLK)];                                                           \
        } else {                                                                                        \
            _Pragma("unroll") for (int i = 0; i < 16; ++i) CREG[i] = 0;                                 \
            PREG = 0u;                                                                                  \
        }                                                                                               \
    } while (0)

    // Filter epilogue of one block of 32 queries x 32 rows (accumulators VEC).
#define LPQ_EPI(VEC, NBI, ROWBASE, PWORD)                                                               \
    do {                                                                                                \
        const int nb = (NBI);                                                                           \
        const v16i v = (VEC);                                                                           \
        if (SEED && GR == 16) {                                                                         \
            _Pragma("unroll") for (int r = 0; r < GR; ++r) gm[nb][r] = max(gm[nb][r], v[r]);            \
        } else {                                                                                        \
            int m = max(max(v[0], v[1]), v[2]);                                                         \
            m = max(max(m, v[3]), v[4]);                                                                \
            m = max(max(m, v[5]), v[6]);                                                                \
            m = max(max(m, v[7]), v[8]);                                                                \
            m = max(max(m, v[9]), v[10]);                                                               \
            m = max(max(m, v[11]), v[12]);                                                              \
            m = max(max(m, v[13]), v[14]);                                                              \
            m = max(m, v[15]);                                                                          \
            if (SEED) {                                                                                 \
                gm[nb][0] = max(gm[nb][0], m);                                                          \
            } else {                                                                                    \
                bool trip = m >= thr[nb];                                                               \
                unsigned long long mask = __ballot(trip);                                               \
                LPQ_SCHED_CHAIN();                                                                      \
                if (__builtin_expect(mask != 0, TRIP_INLINE)) {   /* see TRIP_INLINE */                 \
                    if (qcnt + __popcll(mask) > QCAP) { /* no room: this wave drains alone */           \
                        if (LPQ_DRY(a) < 5) drain_queue<L2, KCAP, LK>(w, qcnt, re, lane, lst, seedC, cbase, qstride, o.Cs); \
                        qcnt = 0;                                                                       \
                        _Pragma("unroll") for (int j = 0; j < NB; ++j) thr[j] = w.thrE[j * 32 + col];   \
                        LPQ_LGKM_SETTLED();                                                             \
                        trip = m >= thr[nb];                                                            \
                        mask = __ballot(trip);                                                          \
                    }                                                                                   \
                    if (mask) {                                                                         \
                        const int below = __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),             \
                                                                    __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u)); \
                        if (trip && LPQ_DRY(a) != 5) {                                                   \
                            const int slot = qcnt + below;                                              \
                            v4i *dst_ = reinterpret_cast<v4i *>(w.qvals + slot * 16);                   \
                            _Pragma("unroll") for (int g = 0; g < 4; ++g)                               \
                                dst_[g] = v4i{v[4 * g], v[4 * g + 1], v[4 * g + 2], v[4 * g + 3]};      \
                            w.qmeta[slot] = v4i{(ROWBASE), (int)(PWORD), (nb * 32 + col) | (half << 8), 0}; \
                        }                                                                               \
                        qcnt += __popcll(mask);                                                         \
                    }                                                                                   \
                }                                                                                       \
            }                                                                                           \
        }                                                                                               \
    } while (0)

#define LPQ_CHAIN(NBI, AREG, CREG)                                                                      \
    _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                                   \
        acc[NBI] = __builtin_amdgcn_mfma_i32_32x32x32_i8(AREG[ks], B[NBI][ks], ks == 0 ? CREG : acc[NBI], 0, 0, 0)

    // Order of the contraction and of the filter epilogue.  Each block of 32 queries gets its KS
    // matrix instructions as one chain (dependent instructions of a chain issue back to back), and
    // the epilogue of a block is placed one chain later, so that its vector instructions run while
    // the next chain is in the matrix core; the last block's accumulators are carried over and
    // tested after the first chain of the NEXT 32-row block.  Against k-step-major order with the
    // four epilogues at the end this measured 5.4 % faster on the benchmark workload (1.347 ->
    // 1.274 ms per 10 000 queries) and needs 29 fewer registers (accumulators live shorter).  The
    // seeding pass tests the last block at once: its segment maxima are flushed at stage boundaries.
    v16i carry_acc = {};
    int carry_rowbase = 0;
    unsigned carry_p = 0;
    bool have_carry = false;
#define LPQ_BLOCK(TT, BLK, AREG, CREG, PREG)                                                            \
    do {                                                                                                \
        v16i acc[NB];                                                                                   \
        const unsigned PREG_ = (PREG);                                                                  \
        const int rowbase = (int)(rs + (int64_t)(TT) * sstride + (BLK) * 32);                           \
        LPQ_CHAIN(0, AREG, CREG);                                                                       \
        if (have_carry) LPQ_EPI(carry_acc, NB - 1, carry_rowbase, carry_p);                             \
        _Pragma("unroll") for (int nbi = 1; nbi < NB; ++nbi) {                                          \
            LPQ_CHAIN(nbi, AREG, CREG);                                                                 \
            LPQ_EPI(acc[nbi - 1], nbi - 1, rowbase, PREG_);                                             \
        }                                                                                               \
        if (SEED) {                                                                                     \
            LPQ_EPI(acc[NB - 1], NB - 1, rowbase, PREG_);                                               \
        } else {                                                                                        \
            carry_acc = acc[NB - 1]; carry_rowbase = rowbase; carry_p = PREG_; have_carry = true;       \
        }                                                                                               \
    } while (0)

    // Where the compiler lays out the path a passing block takes: out of the loop (expected never)
    // or in line.  In line measured 2 % faster at k = 100 on 128-byte rows with 128 queries per wave
    // (a third of the epilogues pass there; 1.254 -> 1.229 ms) and the same at k = 10, but 2.6 %
    // slower on 96-byte rows and 1 % slower in the 64-queries-per-wave kernels: in line for that tile only.
    constexpr int TRIP_INLINE = (KS == 4 && NB == 4) ? 1 : 0;
    int T = (re > rs) ? (int)((re - rs + RS - 1) / RS) : 0;
    if (pieces) {
        T = o.piece_stages;
    } else if (ILV) {   // stages s, s + S, s + 2S, ... of the ceil(rows / RS) stages of the corpus
        const int64_t all = (row1 - row0 + RS - 1) / RS;
        T = (all > s) ? (int)((all - s + S - 1) / S) : 0;
    } else if (SEED && o.stage_stride) {   // split_rows / RS stages, as far as their first rows are real items
        const int64_t left = (row1 > rs) ? (row1 - rs + sstride - 1) / sstride : 0;
        T = (int)(left < split_rows / RS ? left : split_rows / RS);
    }

    // Seeding pass: the GR group maxima of (segment g of this split, lane half) go to
    // gmax[q][(((s*SEG + g) [* NW + wave]) * 2 + half) * GR + r].
    const int G = S * SEG * 2 * GR * (RSPLIT ? NW : 1);
#define LPQ_FLUSH_SEGMENT(SEGIDX)                                                                       \
    do {                                                                                                \
        int lane_ = lane;   /* addresses are formed here, not carried through the loop in registers */ \
        if (REFORM) LPQ_OPAQUE(lane_);                                                                  \
        _Pragma("unroll") for (int nb = 0; nb < NB; ++nb) {                                             \
            int32_t *dst_ = gmax + (size_t)(q_first + nb * 32 + (lane_ & 31)) * G +                     \
                ((((size_t)s * SEG + (SEGIDX)) * (RSPLIT ? NW : 1) + (RSPLIT ? wave : 0)) * 2 + (lane_ >> 5)) * GR; \
            _Pragma("unroll") for (int r = 0; r < GR; ++r) {                                            \
                dst_[r] = gm[nb][r];                                                                    \
                gm[nb][r] = INT32_MIN;                                                                  \
            }                                                                                           \
        }                                                                                               \
    } while (0)
    if (SEED) {   // segments this split never reaches keep the neutral value
        for (int g = 0; g < SEG; ++g) LPQ_FLUSH_SEGMENT(g);
    }

    // Query fragments (and the stores above) have completed before any copy is issued, so from
    // here on only async copies are outstanding on the vector-memory counter.
    __builtin_amdgcn_s_waitcnt(0x0F70);

    // Software pipeline.  While block (t, 0) is in the matrix core the operands of (t, 1) are read
    // from LDS; while (t, 1) is in the matrix core the operands of (t+1, 0) are read.  The
    // workgroup barrier sits in front of block (t, 1): by then every wave has finished READING
    // stage t (its last LDS reads were waited for), so the ring slot of stage t can be refilled
    // with stage t + NST, and stage t+1 is known to have landed.
    if constexpr (RSPLIT) {
        // One 32-row block per wave and stage, no workgroup barrier: the wave waits for its own
        // copies of stage t, refills the slot it finished reading one step ago, and computes.
        v4i A0[KS];
        v16i C0;
        unsigned P0 = 0;
        for (int st = 0; st < NST - 1 && st < T; ++st) LPQ_ISSUE(st);
        for (int t = 0; t < T; ++t) {
            // stages issued so far: 0 .. min(T-1, t+NST-2); wait until stage t has landed
            const int newer = (T - 1 < t + NST - 2 ? T - 1 : t + NST - 2) - t;
            wait_vmcnt(newer * lpt);
            if (t + NST - 1 < T) LPQ_ISSUE(t + NST - 1);   // into the slot of stage t-1
            LPQ_LOAD_BLOCK(t, wave, A0, C0, P0);
            LPQ_BLOCK(t, wave, A0, C0, P0);
            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // my reads of stage t are complete
            if (SEED) {
                const int seg = (int)((int64_t)t * SEG / T), seg_next = (int)((int64_t)(t + 1) * SEG / T);
                if (t + 1 == T || seg_next != seg) {
                    LPQ_FLUSH_SEGMENT(seg);
                    __builtin_amdgcn_s_waitcnt(0x0F70);
                }
            }
        }
    } else {
        v4i A0[KS], A1[KS];
        v16i C0, C1;
        unsigned P0 = 0, P1 = 0;
        const bool abl_nodma = LPQ_DRY(a) == 3 || LPQ_DRY(a) == 4, abl_nobar = LPQ_DRY(a) == 2 || LPQ_DRY(a) == 4;   // timing ablations
        const int primed = T < NST ? T : NST;
        if (!abl_nodma) for (int st = 0; st < primed; ++st) LPQ_ISSUE(st);
        if (T > 0) {
            wait_vmcnt((primed - 1) * lpt);
            __syncthreads();
            LPQ_LOAD_BLOCK(0, 0, A0, C0, P0);
        }
        // Drain requests are acted on one stage late: the flags written before the barrier of
        // stage t are read right after it, but only looked at after the barrier of stage t + 1, so
        // the LDS round trip is off the critical path (the queue keeps room for that extra stage).
        v4i fl0 = {0, 0, 0, 0}, fl1 = {0, 0, 0, 0};
        for (int t = 0; t < T; ++t) {
            LPQ_LOAD_BLOCK(t, 1, A1, C1, P1);
            LPQ_BLOCK(t, 0, A0, C0, P0);
            if constexpr (BIG) {
                LPQ_LOAD_BLOCK(t, 2, A0, C0, P0);
                LPQ_BLOCK(t, 1, A1, C1, P1);
                LPQ_LOAD_BLOCK(t, 3, A1, C1, P1);
                LPQ_BLOCK(t, 2, A0, C0, P0);
            }

            asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");   // my reads of stage t are complete
            if (!SEED && lane == 0) flags[(t & 1) * 8 + wave] = qcnt >= TRIG;
            if (t + 1 < T && !abl_nodma) {
                // stages issued so far: 0 .. min(T-1, t+NST-1); stage t+1 must have landed
                const int last = T - 1 < t + NST - 1 ? T - 1 : t + NST - 1;
                wait_vmcnt((last - (t + 1)) * lpt);
            }
            if (!abl_nobar) __syncthreads();
            if (t + NST < T && !abl_nodma) LPQ_ISSUE(t + NST);   // refills the slot of stage t
            if (!SEED) {
                int any = fl0[0] | fl0[1] | fl0[2] | fl0[3];
                if (NW > 4) any |= fl1[0] | fl1[1] | fl1[2] | fl1[3];
                fl0 = *reinterpret_cast<const v4i *>(flags + (t & 1) * 8);
                if (NW > 4) fl1 = *reinterpret_cast<const v4i *>(flags + (t & 1) * 8 + 4);
                if (any) {   // same answer in every wave of the workgroup: drain together
                    if (LPQ_DRY(a) < 5) drain_queue<L2, KCAP, LK>(w, qcnt, re, lane, lst, seedC, cbase, qstride, o.Cs);
                    qcnt = 0;
#pragma unroll
                    for (int j = 0; j < NB; ++j) thr[j] = w.thrE[j * 32 + col];
                    LPQ_LGKM_SETTLED();
                }
            }
            if (t + 1 < T) LPQ_LOAD_BLOCK(t + 1, 0, A0, C0, P0);
            LPQ_BLOCK(t, BIG ? 3 : 1, A1, C1, P1);

            if (SEED) {   // close a segment when the next stage belongs to the next one
                const int seg = (int)((int64_t)t * SEG / T), seg_next = (int)((int64_t)(t + 1) * SEG / T);
                if (t + 1 == T || seg_next != seg) {
                    LPQ_FLUSH_SEGMENT(seg);
                    __builtin_amdgcn_s_waitcnt(0x0F70);   // keep the counter to async copies only
                }
            }
        }
    }
    if (!SEED && have_carry) LPQ_EPI(carry_acc, NB - 1, carry_rowbase, carry_p);
#undef LPQ_ISSUE
#undef LPQ_EPI
#undef LPQ_CHAIN
#undef LPQ_LOAD_BLOCK
#undef LPQ_BLOCK
#undef LPQ_FLUSH_SEGMENT
#undef LPQ_OPAQUE

    if (COLLECT) {
        if (LPQ_DRY(a) < 5) drain_queue<L2, KCAP, LK>(w, qcnt, re, lane, lst, seedC, cbase, qstride, o.Cs);
        wave_lds_sync();
        for (int i = lane; i < QW; i += 64) {
            const int64_t gq = q_first + i;
            if (gq < a.nq) o.ccnt[(size_t)gq * SS + sub] = w.mbox[i];
        }
    } else if (!SEED) {
        if (LPQ_DRY(a) < 5) drain_queue<L2, KCAP, LK>(w, qcnt, re, lane, lst, seedC, cbase, qstride, o.Cs);
        if constexpr (RSPLIT && KCAP > 0) {
            // The waves hold lists of the SAME 64 queries over different rows: waves 1.. publish
            // theirs in the (now idle) ring and wave 0 folds them into its own.
            cand_t *xl = reinterpret_cast<cand_t *>(ring);
            __syncthreads();
            if (wave > 0) {
#pragma unroll
                for (int i = 0; i < LK; ++i) xl[((wave - 1) * LK + i) * 64 + lane] = lst[i];
            }
            __syncthreads();
            if (wave == 0) {
                for (int i = 0; i < (NW - 1) * LK; ++i)   // pinned slots (index % KCAP < KCAP - k) are not candidates
                    reglist_insert<LK>(lst, xl[i * 64 + lane], i % LK >= LK - k);
            }
        }
        const int64_t gq = q_first + lane;
        if (gq < a.nq && (!RSPLIT || wave == 0)) {
            cand_t *out = lists_out + ((size_t)gq * S + s) * k;
#pragma unroll
            for (int i = 0; i < LK; ++i)
                if (i >= LK - k) out[i - (LK - k)] = lst[i];   // pinned slots are skipped; empty ones are CAND_NONE
        }
    }
}

// ---- rows of 384 to 1536 bytes, and large batches on rows of 192 and 256 bytes -----------------
// The collecting scan and its seeding pass for rows whose operands no longer fit the scheme above
// (query fragments AND two row blocks' worth of corpus fragments in registers).  What changes:
//   - a wave holds the fragments of 32 queries (rows of 768, 1024 or 1536 bytes), 64 (384 or 512
//     bytes) or 128 (192 or 256 bytes): 128 registers at most, 192 on rows of 1536 bytes;
//   - a stage is one block of 32 rows (two where an eight-wave workgroup has the LDS for it) by one
//     segment of the row (the whole row up to 512 bytes, else a half or a third), 6 to 32 KB, in a ring of three
//     to six; the accumulators of a row block live across its segments, are seeded when its first
//     segment starts and filtered when its last one ends;
//   - corpus fragments come from LDS two to four k-steps at a time, one group ahead of the matrix
//     instructions that use them; the group that crosses into the next stage is read right after the
//     workgroup barrier that says the stage has landed.
// Chunks (16 bytes) of a row segment are swizzled inside aligned groups of 2^SWB chunks: with the
// row stride of 512 bytes (a multiple of the 256 bytes the 64 banks cover) the low four bits of the
// row number do it; with 384 bytes odd rows start half way round the banks, so three bits taken
// from bit 1 up give 16 consecutive rows 16 different bank groups as well.
// (Segments of 256 bytes behave like 512, and with 192 bytes a row starts at one of four places
// round the banks, so two bits taken from bit 2 up do it, in groups of four chunks.)
template <int CPS>
__device__ __forceinline__ int long_slot(int c, int r)
{
    constexpr int SWB = CPS % 16 == 0 ? 4 : (CPS % 8 == 0 ? 3 : 2), MASK = (1 << SWB) - 1;
    const int sw = SWB == 4 ? (r & 15) : (SWB == 3 ? ((r >> 1) & 7) : ((r >> 2) & 3));
    return (c & ~MASK) | ((c ^ sw) & MASK);
}

// blocks of 32 queries per wave: as many as 128 registers of query fragments allow
constexpr int long_nb(int kseg, int nseg) { return nseg >= 2 ? 1 : (kseg >= 12 ? 2 : 4); }
// rows per stage: two row blocks where one workgroup has the CU's LDS to itself (eight waves; the
// seeding pass samples the same stages): twice the matrix instructions per barrier, copy wait and
// loop turn
// (not the seeding pass of rows up to 256 bytes: with 128 queries per wave and no branch between
// its row blocks the compiler schedules both as one region and spills 24 to 45 registers)
constexpr int long_rs(int kseg, bool seed, int nw) { return (nw == 8 && !(seed && kseg <= 8)) ? 64 : 32; }
constexpr int long_nst(int kseg, int nw, int rs)
{
    return nw == 4 ? (kseg <= 8 ? 4 : 3) : (rs == 64 ? (kseg == 6 ? 5 : (kseg == 16 ? 3 : 4)) : (kseg <= 12 ? 6 : 5));
}
constexpr size_t long_lds_bytes(int kseg, int nb, bool seed, int nw, int rs)
{
    return (size_t)long_nst(kseg, nw, rs) * rs * kseg * 32 + (size_t)long_nst(kseg, nw, rs) * (rs + 4) * 4 + 64 +
           (seed ? 0 : nw * waveq_bytes(nb * 32));
}

template <int KSEG, int NSEG, bool L2, bool SEED, int NW>
__global__ __launch_bounds__(NW * 64, NW == 4 ? 2 : 1) void search_long_kernel(
    SearchArgs a, int64_t row0, int64_t row1, int S, int64_t split_rows, int qtiles, MfmaIo o)
{
    extern __shared__ __align__(16) unsigned char smem[];
    static_assert(((KSEG == 12 || KSEG == 16) && (NSEG == 1 || NSEG == 2)) || ((KSEG == 6 || KSEG == 8) && NSEG == 1) ||
                  (KSEG == 16 && NSEG == 3), "rows of 192, 256, 384, 512, 768, 1024 or 1536 bytes");
    static_assert(NW == 4 || NW == 8, "four waves (two workgroups per CU) or eight (one)");
    constexpr int NB = long_nb(KSEG, NSEG);    // blocks of 32 queries per wave
    constexpr int QW = NB * 32, QT = NW * QW;
    constexpr int KTOT = KSEG * NSEG;          // k-steps (32 bytes) per row
    constexpr int ROWB = KTOT * 32, SEGB = KSEG * 32;
    constexpr int CPS = SEGB / 16;             // chunks per row segment
    constexpr int RS = long_rs(KSEG, SEED, NW);   // rows per stage
    constexpr int BPS = RS / 32;               // row blocks per stage
    constexpr int NST = long_nst(KSEG, NW, RS);
    constexpr int STAGE_BYTES = RS * SEGB;
    constexpr int NI = RS * CPS / 64;          // copy instructions per stage: wave w issues w, w + NW, ...
    constexpr int IPW = (NI + NW - 1) / NW;    // ... at most this many
    constexpr int AUX_INTS = RS + 4;           // accumulator seeds of the 32 rows, then their parity word
    constexpr int GS = KSEG == 6 ? 3 : ((KSEG == 8 || NSEG == 3) ? 2 : 4);   // k-steps per group of fragments (each feeds NB matrix instructions)
    constexpr int NG = KSEG / GS;              // groups per segment
    constexpr int PER = CPS % 16 == 0 ? 8 : (CPS % 8 == 0 ? 4 : 2);   // k-steps after which a lane's swizzle pattern repeats
    static_assert((NST - 1) * (IPW + 1) <= 63, "wait_vmcnt covers 0..63");

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col = lane & 31, half = lane >> 5;

    // the same XCD-aware order of (split, query tile) pairs as the kernel above
    const int total = qtiles * S;
    const int per = total / 8;
    const int b = blockIdx.x;
    const int wk = (a.work_order != 3 && b < per * 8) ? (b % 8) * per + b / 8 : b;
    const int s = (a.work_order == 2) ? wk % S : wk / qtiles;
    const int qt = (a.work_order == 2) ? wk / S : wk % qtiles;

    // Row blocks of this split.  Collecting scan: blocks s, s + S, s + 2S, ... of the corpus, so that
    // a query's candidates spread evenly over the splits' regions.  Seeding pass: split_rows / 32
    // blocks starting at row0 + s * split_stride, stage_stride rows apart (adjacent without a stride),
    // as far as their first rows are real items.
    int RB;
    int64_t rs, bstride;
    if (!SEED) {
        const int64_t all = (row1 - row0 + RS - 1) / RS;
        RB = (all > s) ? (int)((all - s + S - 1) / S) : 0;
        rs = row0 + (int64_t)s * RS;
        bstride = (int64_t)S * RS;
    } else {
        rs = row0 + (int64_t)s * o.split_stride;
        bstride = o.stage_stride ? o.stage_stride : RS;
        const int64_t left = (row1 > rs) ? (row1 - rs + bstride - 1) / bstride : 0;
        RB = (int)(left < split_rows / RS ? left : split_rows / RS);
    }
    const int T = RB * NSEG;
    const int64_t re = row1;

    unsigned char *ring = smem;
    int *aux = (int *)(smem + NST * STAGE_BYTES);
    int *flags = aux + NST * AUX_INTS;           // [8] joint-drain requests, one per wave (16 words are set aside)
    const WaveQ w = carve_waveq((unsigned char *)(flags + 16) + (size_t)wave * waveq_bytes(QW), QW);
    const int64_t q_first = (int64_t)qt * QT + wave * QW;

    if constexpr (!SEED) {
        if (a.redo_flags) {   // a further round: only if the flagged queries are many, and only tiles that hold one
            if (*a.redo_count <= a.redo_min) return;   // the same answer in every thread of the grid
            const int64_t t0 = (int64_t)qt * QT;
            int mine = 0;
            for (int64_t qq = t0 + tid; qq < t0 + QT && qq < a.nq; qq += NW * 64) mine |= a.redo_flags[qq];
            int *vote = reinterpret_cast<int *>(ring);   // the ring is still unused
            if (tid == 0) *vote = 0;
            __syncthreads();
            if (mine) atomicOr(vote, 1);
            __syncthreads();
            const int any = *vote;
            __syncthreads();   // everyone has read the vote before the ring is filled
            if (!any) return;  // the same answer in every thread of the workgroup
        }
    }

    cand_t lst[1] = {0};
    const cand_t seedC = 0;
    cand_t *cbase = SEED ? nullptr : o.cbuf + ((size_t)q_first * S + s) * o.Cs;
    const size_t qstride = (size_t)S * o.Cs;
    if (!SEED) {
        for (int i = lane; i < QW; i += 64) {
            const int64_t gq = q_first + i;
            const cand_t sc = gq < a.nq ? (o.seeds ? o.seeds[gq] : CAND_NONE) : 0;
            w.thrC[i] = sc;
            w.thrE[i] = thr_e(sc);
            w.mbox[i] = 0;
        }
    }
    wave_lds_sync();

    v4i B[NB][KTOT];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
        for (int ks = 0; ks < KTOT; ++ks)
            B[nb][ks] = *reinterpret_cast<const v4i *>(a.qcodes + (q_first + nb * 32 + col) * a.d_pad + ks * 32 + half * 16);
    int thr[NB], gm[NB];
#pragma unroll
    for (int nb = 0; nb < NB; ++nb) {
        thr[nb] = SEED ? INT32_MAX : w.thrE[nb * 32 + col];
        gm[nb] = INT32_MIN;
    }
    int qcnt = 0;
    // Byte offset, inside a stage, of this lane's fragment of k-step ks (of the segment): the chunk
    // 2 ks + half sits in slot long_slot(2 ks + half, col), which differs from the slot of k-step 0
    // only in the bits ks % PER sets (the row's start has those address bits clear), so one register
    // and an exclusive-or with a constant per read replace a table of PER offsets:
    // offset(ks) = (a_base ^ ((ks % PER) << 5)) + (ks / PER) * PER * 32.
    const int a_base = col * SEGB + long_slot<CPS>(half, col) * 16;
    static_assert(SEGB % (PER * 32) == 0, "a row starts on a multiple of the swizzle group");

    // Stage loader: LDS position p (16 bytes) of a stage = (row p / CPS, slot p % CPS); copy instruction
    // i of a stage fills positions [64 i, 64 i + 64), each lane fetching the chunk that belongs in its
    // slot, and wave w issues instructions w, w + NW, ...
    const unsigned ring_lds = lds_offset(ring), aux_lds = lds_offset(aux);
    const int mine = (NI - wave + NW - 1) / NW;         // copy instructions of this wave
    const int lpt = mine + ((L2 && wave < 2) ? 1 : 0);  // copies this wave issues per stage
    int src_off[IPW];
#pragma unroll
    for (int j = 0; j < IPW; ++j) {
        const int p = (wave + j * NW) * 64 + lane;
        const int r = p / CPS, sl = p % CPS;
        src_off[j] = r * ROWB + long_slot<CPS>(sl, r) * 16;   // the swizzle is its own inverse
    }
#define LPQL_ISSUE(ST, SLOT)                                                                            \
    do {                                                                                                \
        const int st_ = (ST), slot_ = (SLOT);                                                           \
        const int64_t r0_ = rs + (int64_t)(st_ / NSEG) * bstride;                                       \
        const int8_t *src_ = a.codes + r0_ * ROWB + (st_ % NSEG) * SEGB;                                \
        _Pragma("unroll") for (int j = 0; j < IPW; ++j)                                                 \
            if (NI % NW == 0 || j < mine) {                                                             \
                int near_ = src_off[j];   /* one register each: the 64-bit address is formed here, not */ \
                asm volatile("" : "+v"(near_));   /* carried through the loop (and spilled) as a pair  */ \
                async_copy16(src_ + near_,                                                              \
                             __builtin_amdgcn_readfirstlane(ring_lds + slot_ * STAGE_BYTES + (wave + j * NW) * 1024)); \
            }                                                                                           \
        if (L2 && wave == 0) {                                                                          \
            if (lane < RS) async_copy4(a.cinit + r0_ + lane, aux_lds + slot_ * AUX_INTS * 4);           \
        } else if (L2 && wave == 1) {                                                                   \
            if (lane < BPS) async_copy4(a.parity + r0_ / 32 + lane, aux_lds + (slot_ * AUX_INTS + RS) * 4); \
        }                                                                                               \
    } while (0)

    // fragments of group G (k-steps GS G .. GS G + GS - 1 of the segment) of row block BLK of the stage in ring slot SLOT
#define LPQL_LOAD_GROUP(SLOT, BLK, G, AREG)                                                             \
    do {                                                                                                \
        const unsigned char *sb_ = ring + (size_t)(SLOT) * STAGE_BYTES + (BLK) * 32 * SEGB;             \
        _Pragma("unroll") for (int i = 0; i < GS; ++i) {                                                \
            const int ks_ = (G) * GS + i;                                                               \
            AREG[i] = *reinterpret_cast<const v4i *>(sb_ + (a_base ^ ((ks_ % PER) << 5)) + (ks_ / PER) * (PER * 32)); \
        }                                                                                               \
    } while (0)
    // accumulator seeds and parity word of row block BLK of the stage in ring slot SLOT
#define LPQL_LOAD_SEEDS(SLOT, BLK, CREG, PREG)                                                          \
    do {                                                                                                \
        if (L2) {                                                                                       \
            const int *cb_ = aux + (SLOT) * AUX_INTS;                                                   \
            _Pragma("unroll") for (int g = 0; g < 4; ++g) {                                             \
                const v4i v_ = *reinterpret_cast<const v4i *>(cb_ + (BLK) * 32 + 8 * g + 4 * half);     \
                CREG[4 * g + 0] = v_[0]; CREG[4 * g + 1] = v_[1];                                       \
                CREG[4 * g + 2] = v_[2]; CREG[4 * g + 3] = v_[3];                                       \
            }                                                                                           \
            PREG = (unsigned)cb_[RS + (BLK)];                                                           \
        } else {                                                                                        \
            _Pragma("unroll") for (int i = 0; i < 16; ++i) CREG[i] = 0;                                 \
            PREG = 0u;                                                                                  \
        }                                                                                               \
    } while (0)

    // filter epilogue of one block of 32 queries x 32 rows, as in the kernel above
#define LPQL_EPI(VEC, NBI, ROWBASE, PWORD)                                                              \
    do {                                                                                                \
        const int nb = (NBI);                                                                           \
        const v16i v = (VEC);                                                                           \
        int m = max(max(v[0], v[1]), v[2]);                                                             \
        m = max(max(m, v[3]), v[4]);                                                                    \
        m = max(max(m, v[5]), v[6]);                                                                    \
        m = max(max(m, v[7]), v[8]);                                                                    \
        m = max(max(m, v[9]), v[10]);                                                                   \
        m = max(max(m, v[11]), v[12]);                                                                  \
        m = max(max(m, v[13]), v[14]);                                                                  \
        m = max(m, v[15]);                                                                              \
        if (SEED) {                                                                                     \
            gm[nb] = max(gm[nb], m);                                                                    \
        } else {                                                                                        \
            bool trip = m >= thr[nb];                                                                   \
            unsigned long long mask = __ballot(trip);                                                   \
            if (__builtin_expect(mask != 0, 0)) {                                                       \
                if (qcnt + __popcll(mask) > QCAP) {   /* no room: this wave drains alone */             \
                    drain_queue<L2, 0, 1>(w, qcnt, re, lane, lst, seedC, cbase, qstride, o.Cs);         \
                    qcnt = 0;                                                                           \
                }                                                                                       \
                const int below = __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32),                     \
                                                            __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u)); \
                if (trip) {                                                                             \
                    const int slot = qcnt + below;                                                      \
                    v4i *dst_ = reinterpret_cast<v4i *>(w.qvals + slot * 16);                           \
                    _Pragma("unroll") for (int g = 0; g < 4; ++g)                                       \
                        dst_[g] = v4i{v[4 * g], v[4 * g + 1], v[4 * g + 2], v[4 * g + 3]};              \
                    w.qmeta[slot] = v4i{(ROWBASE), (int)(PWORD), (nb * 32 + col) | (half << 8), 0};     \
                }                                                                                       \
                qcnt += __popcll(mask);                                                                 \
            }                                                                                           \
        }                                                                                               \
    } while (0)

    // Seeding pass: the group maximum of (segment g of this split, lane half) goes to
    // gmax[q][(s * SEG + g) * 2 + half], the layout the kernel above uses.
    const int SEG = o.SEG;
    const int G = S * SEG * 2;
#define LPQL_FLUSH_SEGMENT(SEGIDX)                                                                      \
    do {                                                                                                \
        int lane_ = lane;   /* likewise: the addresses are formed when a segment closes */              \
        asm volatile("" : "+v"(lane_));                                                                 \
        _Pragma("unroll") for (int nb = 0; nb < NB; ++nb) {                                             \
            o.gmax[(size_t)(q_first + nb * 32 + (lane_ & 31)) * G + ((size_t)s * SEG + (SEGIDX)) * 2 + (lane_ >> 5)] = gm[nb]; \
            gm[nb] = INT32_MIN;                                                                         \
        }                                                                                               \
    } while (0)
    if (SEED) {   // segments this split never reaches keep the neutral value
        for (int g = 0; g < SEG; ++g) LPQL_FLUSH_SEGMENT(g);
    }

    // Query fragments (and the stores above) have completed before any copy is issued, so from
    // here on only async copies (and appended candidates) are outstanding on the vector-memory counter.
    __builtin_amdgcn_s_waitcnt(0x0F70);

    // Seeds and parity word of a row block are read along with its first fragment group, one group
    // ahead - except where the query fragments fill all 128 registers they may have and the 16 more
    // are not there: the block then reads its seeds as it starts.
    constexpr bool SEEDS_AHEAD = KTOT * NB * 4 < 128;
    v4i An[GS];          // the group read ahead
    v16i Cn;             // seeds and parity word of the row block that starts next
    unsigned Pn = 0;
    const int primed = T < NST ? T : NST;
    for (int st = 0; st < primed; ++st) LPQL_ISSUE(st, st);
    int slot = 0;        // ring slot of stage t
    if (T > 0) {
        wait_vmcnt((primed - 1) * lpt);
        __syncthreads();
        LPQL_LOAD_GROUP(0, 0, 0, An);
        if (SEEDS_AHEAD) LPQL_LOAD_SEEDS(0, 0, Cn, Pn);
    }
    int t = 0;
    for (int rb = 0; rb < RB; ++rb) {   // rb: a group of RS rows = BPS row blocks; its NSEG stages follow each other
        v16i acc[BPS][NB];
        v16i Cc;
        unsigned Pc[BPS];
#pragma unroll
        for (int seg = 0; seg < NSEG; ++seg, ++t) {
#pragma unroll
            for (int blk = 0; blk < BPS; ++blk) {
#pragma unroll
                for (int g = 0; g < NG; ++g) {
                    v4i Ac[GS];
#pragma unroll
                    for (int i = 0; i < GS; ++i) Ac[i] = An[i];
                    if (seg == 0 && g == 0) {
                        if (SEEDS_AHEAD) { Cc = Cn; Pc[blk] = Pn; }
                        else LPQL_LOAD_SEEDS(slot, blk, Cc, Pc[blk]);   // the stage's slot is refilled only after its last group
                    }
                    if (g + 1 < NG) {
                        LPQL_LOAD_GROUP(slot, blk, g + 1, An);
                    } else if (blk + 1 < BPS) {   // on to the next row block of the same stage
                        LPQL_LOAD_GROUP(slot, blk + 1, 0, An);
                        if (SEEDS_AHEAD && seg == 0) LPQL_LOAD_SEEDS(slot, blk + 1, Cn, Pn);
                    } else {
                        // the last group of stage t is in registers once the LDS counter is down: this wave
                        // is done reading the stage
                        // (the matrix instructions of the group before are issued first: they run meanwhile)
                        __builtin_amdgcn_sched_barrier(0);
                        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
                        // every fourth stage the waves tell each other whether a queue is half full, and
                        // if one is, all drain together (a wave whose queue overflows in between drains alone)
                        const bool xchg = !SEED && (t & 3) == 3;
                        if (xchg && lane == 0) flags[wave] = qcnt >= TRIG;
                        if (t + NST - 1 < T) {
                            // stages 0 .. t+NST-1 have been issued and stage t+1 must have landed: all but
                            // the copies of the NST-2 newest stages (a constant count per wave, without the
                            // run-time dispatch of wait_vmcnt)
                            if (lpt == IPW) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NST - 2) * IPW));
                            else if (lpt == IPW + 1) __builtin_amdgcn_s_waitcnt(vmcnt_imm((NST - 2) * (IPW + 1)));
                            else wait_vmcnt((NST - 2) * lpt);
                        } else if (t + 1 < T) {   // the tail: stages up to T-1 have been issued
                            wait_vmcnt((T - 1 - (t + 1)) * lpt);
                        }
                        __syncthreads();
                        if (t + NST < T) LPQL_ISSUE(t + NST, slot);   // refills the slot of stage t
                        if (xchg) {   // (the next exchange is four barriers away: no wave can overwrite a flag early)
                            const v4i fl0 = *reinterpret_cast<const v4i *>(flags);
                            int any = fl0[0] | fl0[1] | fl0[2] | fl0[3];
                            if (NW > 4) {
                                const v4i fl1 = *reinterpret_cast<const v4i *>(flags + 4);
                                any |= fl1[0] | fl1[1] | fl1[2] | fl1[3];
                            }
                            if (any) {
                                drain_queue<L2, 0, 1>(w, qcnt, re, lane, lst, seedC, cbase, qstride, o.Cs);
                                qcnt = 0;
                            }
                        }
                        const int nslot = slot + 1 == NST ? 0 : slot + 1;
                        if (t + 1 < T) {
                            LPQL_LOAD_GROUP(nslot, 0, 0, An);
                            if (SEEDS_AHEAD && seg + 1 == NSEG) LPQL_LOAD_SEEDS(nslot, 0, Cn, Pn);
                        }
                        slot = nslot;
                    }
#pragma unroll
                    for (int i = 0; i < GS; ++i)
#pragma unroll
                        for (int nb = 0; nb < NB; ++nb)
                            acc[blk][nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                                Ac[i], B[nb][seg * KSEG + g * GS + i], (seg == 0 && g == 0 && i == 0) ? Cc : acc[blk][nb], 0, 0, 0);
                    // Keep the reads of the next group in front of this group's matrix instructions: left
                    // alone, the compiler moves each read down to the instruction that needs it and every
                    // matrix instruction then waits out a full LDS round trip.  The same two groups keep
                    // ALL matrix instructions of the block in front of its first filter epilogue.  That
                    // matters: with the completing group issued query block by query block and each
                    // epilogue one chain later (as in the kernel above) the scheduler put the last
                    // matrix instruction of a chain four instructions before the branch that ends the
                    // epilogue before it, the next epilogue read that chain's first accumulators five
                    // issue slots after it with no wait inserted, and candidates in those rows went
                    // missing now and then (two runs of one binary disagreed).
                    __builtin_amdgcn_sched_group_barrier(0x100, GS, 0);        // the group's LDS reads
                    __builtin_amdgcn_sched_group_barrier(0x008, GS * NB, 0);   // GS * NB matrix instructions
                    if (seg == NSEG - 1 && g == NG - 1) {   // the row block is complete
                        // nothing of the contraction may drift down among the epilogues (see above)
                        __builtin_amdgcn_sched_barrier(0);
                        const int rowbase = (int)(rs + (int64_t)rb * bstride) + blk * 32;
#pragma unroll
                        for (int nbi = 0; nbi < NB; ++nbi) LPQL_EPI(acc[blk][nbi], nbi, rowbase, Pc[blk]);
                    }
                }
            }
        }
        if (SEED) {   // close a segment when the next row block belongs to the next one
            const int sg = (int)((int64_t)rb * SEG / RB), sg_next = (int)((int64_t)(rb + 1) * SEG / RB);
            if (rb + 1 == RB || sg_next != sg) {
                LPQL_FLUSH_SEGMENT(sg);
                __builtin_amdgcn_s_waitcnt(0x0F70);   // keep the counter to async copies only
            }
        }
    }
#undef LPQL_ISSUE
#undef LPQL_LOAD_GROUP
#undef LPQL_LOAD_SEEDS
#undef LPQL_EPI
#undef LPQL_FLUSH_SEGMENT

    if (!SEED) {
        drain_queue<L2, 0, 1>(w, qcnt, re, lane, lst, seedC, cbase, qstride, o.Cs);
        wave_lds_sync();
        for (int i = lane; i < QW; i += 64) {
            const int64_t gq = q_first + i;
            if (gq < a.nq) o.ccnt[(size_t)gq * S + s] = w.mbox[i];
        }
    }
}

// One wave per query: the k-th largest of its G group maxima (duplicates counted) becomes the
// seed threshold.  Each lane keeps E of the values in registers.  Small k: k times the wave takes
// the largest value left and the first lane holding it drops one copy.  Larger k: bisection on
// the value with wave-wide counts.
template <int E>
__global__ __launch_bounds__(256) void seed_finalize_kernel(const int32_t *__restrict__ gmax, int64_t nq, int G, int k,
                                                            cand_t *__restrict__ seeds, int32_t *__restrict__ zero_word)
{
    const int lane = threadIdx.x & 63;
    if (zero_word && blockIdx.x == 0 && threadIdx.x == 0) *zero_word = 0;
    const int64_t q = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (q >= nq) return;                                   // wave-uniform
    int v[E];
#pragma unroll
    for (int e = 0; e < E; ++e) {
        const int i = e * 64 + lane;
        v[e] = (i < G) ? gmax[q * G + i] : INT32_MIN;
    }
    int kth = INT32_MIN;
    if (k <= 24) {
        for (int r = 0; r < k; ++r) {
            int mx = v[0];
#pragma unroll
            for (int e = 1; e < E; ++e) mx = v[e] > mx ? v[e] : mx;
            const int wmx = wave_max_i32(mx);
            kth = wmx;
            const int win = __ffsll((unsigned long long)__ballot(mx == wmx)) - 1;
            bool done = lane != win;
#pragma unroll
            for (int e = 0; e < E; ++e) {
                const bool hit = !done && v[e] == wmx;
                v[e] = hit ? INT32_MIN : v[e];
                done = done || hit;
            }
        }
    } else if (G >= k) {
        // larger k: bisection on the value; the answer is the largest t with #{v >= t} >= k
        int mn = v[0], mx = v[0];
#pragma unroll
        for (int e = 1; e < E; ++e) {
            mn = v[e] < mn ? v[e] : mn;
            mx = v[e] > mx ? v[e] : mx;
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) {
            const int a = __shfl_xor(mn, o, 64), b = __shfl_xor(mx, o, 64);
            mn = a < mn ? a : mn;
            mx = b > mx ? b : mx;
        }
        long long lo = mn, hi = mx;        // #{v >= lo} = all >= k; the answer lies in [lo, hi]
        while (lo < hi) {                  // wave-uniform
            const long long mid = lo + (hi - lo + 1) / 2;
            int cnt = 0;
#pragma unroll
            for (int e = 0; e < E; ++e) cnt += __popcll(__ballot(v[e] >= (int)mid));
            if (cnt >= k) lo = mid; else hi = mid - 1;
        }
        kth = (int)lo;
    }
    // at least k items have E >= kth, hence key <= -2 kth
    if (lane == 0) seeds[q] = (G < k || kth == INT32_MIN) ? CAND_NONE : make_cand(-2 * kth, 0xFFFFFFFFu);
}

size_t lds_bytes(int ks, bool seed, int nw, bool rsplit, int nb, bool pack, bool big = false)
{
    const int cpr = pack ? ks : 2 * ks;
    const int slots = cpr <= 2 ? 2 : (cpr <= 4 ? 4 : (cpr <= 8 ? 8 : 16));
    const int nst = ring_depth(ks, rsplit, pack, big);
    const int rs = rsplit ? 32 * nw : (big ? 128 : 64);
    return (size_t)nst * rs * slots * 16 + (size_t)nst * (rs + 4) * 4 + 64 + (seed ? 0 : nw * waveq_bytes(nb * 32));
}

template <int KS, bool L2, int KCAP, bool SEED, int NW, bool RSPLIT, int NB = 2, bool PACK = false>
hipError_t launch_nw(const SearchArgs &a, int64_t row0, int64_t row1, int S, int64_t split_rows, MfmaIo o, hipStream_t st)
{
    const int qtiles = (int)ceil_div(a.nq, RSPLIT ? NQW : NW * NB * 32);
    const size_t lds = lds_bytes(KS, SEED, NW, RSPLIT, NB, PACK, big_stage(KCAP, SEED, RSPLIT, NB, PACK, KS));
    auto kern = search_mfma_kernel<KS, L2, KCAP, SEED, NW, RSPLIT, NB, PACK>;
    static bool attr_set = false;  // per instantiation
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    kern<<<(unsigned)(qtiles * S), NW * 64, lds, st>>>(a, row0, row1, S, split_rows, qtiles, o);
    return hipGetLastError();
}

// Four waves (256 queries) per workgroup, two workgroups per CU.  Eight-wave workgroups (one per
// CU, half the corpus bytes per contraction) measured slower: the wider barrier costs more than
// the saved L1 traffic.
template <int KS, bool L2, int KCAP, bool SEED>
hipError_t launch_one(const SearchArgs &a, int64_t row0, int64_t row1, int S, MfmaIo o, hipStream_t st)
{
    // rows of a split: a whole number of stages; splits follow each other unless a stride is given
    const int64_t split_rows = o.split_stride ? o.split_stride_rows : round_up(ceil_div(row1 - row0, S), 128);
    if (!o.split_stride) o.split_stride = split_rows;
    if (a.packed) {
        // packed rows: row-split launches (register lists, or the collecting scan for longer lists,
        // and their seeding pass) for up to 64 queries; large batches: the collecting scan (and its
        // seeding pass), 128 queries per wave on rows of up to 64 bytes, 64 on longer ones
        if (a.rsplit) {
            if (a.rs_waves != 4) return hipErrorInvalidValue;
            return launch_nw<KS, L2, KCAP, SEED, 4, true, 2, true>(a, row0, row1, S, split_rows, o, st);
        }
        if constexpr ((KCAP == 0 || SEED) && KS >= 3) {
            if constexpr (KS <= 4) {
                if (a.wave_queries != 128) return hipErrorInvalidValue;
                return launch_nw<KS, L2, KCAP, SEED, 4, false, 4, true>(a, row0, row1, S, split_rows, o, st);
            } else {
                if (a.wave_queries != 64) return hipErrorInvalidValue;
                return launch_nw<KS, L2, KCAP, SEED, 4, false, 2, true>(a, row0, row1, S, split_rows, o, st);
            }
        }
        return hipErrorInvalidValue;
    }
    if constexpr (KS <= 4) {
        if (a.rsplit) {
            if (a.rs_waves != 4) return hipErrorInvalidValue;
            return launch_nw<KS, L2, KCAP, SEED, 4, true>(a, row0, row1, S, split_rows, o, st);
        }
        if constexpr (KCAP == 0 || SEED) {
            if (a.wave_queries == 128) return launch_nw<KS, L2, KCAP, SEED, 4, false, 4>(a, row0, row1, S, split_rows, o, st);
        }
    } else if (a.rsplit) {   // rows of 192 or 256 bytes: two waves per workgroup, 64-row stages (collecting scan and seeding pass)
        if constexpr (KCAP == 0 || SEED) {
            if (a.rs_waves != 2) return hipErrorInvalidValue;
            return launch_nw<KS, L2, KCAP, SEED, 2, true>(a, row0, row1, S, split_rows, o, st);
        }
        return hipErrorInvalidValue;
    }
    return launch_nw<KS, L2, KCAP, SEED, 4, false>(a, row0, row1, S, split_rows, o, st);
}

template <int KS>
hipError_t launch_ks(const SearchArgs &a, int64_t row0, int64_t row1, int S, const MfmaIo &o, hipStream_t st)
{
    const bool l2 = a.metric == LPQ_METRIC_L2SQ;
    if (o.gmax)
        return l2 ? launch_one<KS, true, 1, true>(a, row0, row1, S, o, st)
                  : launch_one<KS, false, 1, true>(a, row0, row1, S, o, st);
    if (o.cbuf)
        return l2 ? launch_one<KS, true, 0, false>(a, row0, row1, S, o, st)
                  : launch_one<KS, false, 0, false>(a, row0, row1, S, o, st);
    if (a.k <= 10)
        return l2 ? launch_one<KS, true, 10, false>(a, row0, row1, S, o, st)
                  : launch_one<KS, false, 10, false>(a, row0, row1, S, o, st);
    return l2 ? launch_one<KS, true, 16, false>(a, row0, row1, S, o, st)
              : launch_one<KS, false, 16, false>(a, row0, row1, S, o, st);
}

// Launches the plan laid out for the long-row scan (its query tile says so).
bool takes_long_scan(const SearchArgs &a)
{
    return mfma_long_rows(a.d_pad, a.nq) && !a.rsplit && !a.packed && a.wave_queries == mfma_long_wave_queries(a.d_pad);
}

// Rows of 384 to 1536 bytes (and large batches on 192 and 256): the collecting scan (o.cbuf) or its seeding pass (o.gmax).
template <int KSEG, int NSEG, bool L2, bool SEED, int NW>
hipError_t launch_long_nw(const SearchArgs &a, int64_t row0, int64_t row1, int S, MfmaIo o, hipStream_t st)
{
    constexpr int NB = long_nb(KSEG, NSEG);
    if (a.rsplit || a.packed || a.wave_queries != NB * 32) return hipErrorInvalidValue;
    const int64_t split_rows = o.split_stride ? o.split_stride_rows : round_up(ceil_div(row1 - row0, S), 128);
    if (!o.split_stride) o.split_stride = split_rows;
    const int qtiles = (int)ceil_div(a.nq, NW * NB * 32);
    auto kern = search_long_kernel<KSEG, NSEG, L2, SEED, NW>;
    static bool attr_set = false;  // per instantiation
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    kern<<<(unsigned)(qtiles * S), NW * 64, long_lds_bytes(KSEG, NB, SEED, NW, long_rs(KSEG, SEED, NW)), st>>>(
        a, row0, row1, S, split_rows, qtiles, o);
    return hipGetLastError();
}

template <int KSEG, int NSEG, bool L2, bool SEED>
hipError_t launch_long_one(const SearchArgs &a, int64_t row0, int64_t row1, int S, const MfmaIo &o, hipStream_t st)
{
    if constexpr (NSEG < 3) {
        if (mfma_long_waves(a.d_pad, a.nq) == 8) return launch_long_nw<KSEG, NSEG, L2, SEED, 8>(a, row0, row1, S, o, st);
    }
    return launch_long_nw<KSEG, NSEG, L2, SEED, 4>(a, row0, row1, S, o, st);
}

template <int KSEG, int NSEG>
hipError_t launch_long(const SearchArgs &a, int64_t row0, int64_t row1, int S, const MfmaIo &o, hipStream_t st)
{
    const bool l2 = a.metric == LPQ_METRIC_L2SQ;
    if (o.gmax)
        return l2 ? launch_long_one<KSEG, NSEG, true, true>(a, row0, row1, S, o, st)
                  : launch_long_one<KSEG, NSEG, false, true>(a, row0, row1, S, o, st);
    if (o.cbuf)
        return l2 ? launch_long_one<KSEG, NSEG, true, false>(a, row0, row1, S, o, st)
                  : launch_long_one<KSEG, NSEG, false, false>(a, row0, row1, S, o, st);
    return hipErrorInvalidValue;   // no register lists beside rows this long
}

hipError_t launch_any(const SearchArgs &a, int64_t row0, int64_t row1, int S, const MfmaIo &o, hipStream_t st)
{
    if (a.nq <= 0 || row1 <= row0) return hipSuccess;
    if (row0 % 128 || o.split_stride % 128) return hipErrorInvalidValue;  // stages and parity words cover aligned blocks
    if (takes_long_scan(a) && (o.gmax || o.cbuf)) {
        switch (a.d_pad / 32) {
        case 6: return launch_long<6, 1>(a, row0, row1, S, o, st);
        case 8: return launch_long<8, 1>(a, row0, row1, S, o, st);
        case 12: return launch_long<12, 1>(a, row0, row1, S, o, st);
        case 16: return launch_long<16, 1>(a, row0, row1, S, o, st);
        case 24: return launch_long<12, 2>(a, row0, row1, S, o, st);
        case 32: return launch_long<16, 2>(a, row0, row1, S, o, st);
        case 48: return launch_long<16, 3>(a, row0, row1, S, o, st);
        default: break;
        }
    }
    switch (a.d_pad / 32) {
    case 2: return launch_ks<2>(a, row0, row1, S, o, st);
    case 3: return launch_ks<3>(a, row0, row1, S, o, st);
    case 4: return launch_ks<4>(a, row0, row1, S, o, st);
    case 6: return launch_ks<6>(a, row0, row1, S, o, st);
    case 8: return launch_ks<8>(a, row0, row1, S, o, st);
    default: return hipErrorInvalidValue;
    }
}

bool shape_ok(int d_pad)
{
    const int ks = d_pad / 32;
    return d_pad % 32 == 0 && (ks == 2 || ks == 3 || ks == 4 || ks == 6 || ks == 8);
}

bool long_shape_ok(int d_pad) { return d_pad == 384 || d_pad == 512 || d_pad == 768 || d_pad == 1024 || d_pad == 1536; }

}  // namespace

int mfma_queries_per_workgroup(int64_t nq, int d_pad, bool wide)
{
    if (long_shape_ok(d_pad)) return mfma_long_waves(d_pad, nq) * mfma_long_wave_queries(d_pad);
    return mfma_row_split(nq, d_pad) ? 64 : (wide ? 512 : 256);
}

// Rows of more than 256 bytes (384, 512, 768 or 1024: the collecting scan and its seeding pass only).
bool mfma_long_rows(int d_pad, int64_t nq)
{
    // Rows of 192 and 256 bytes: the same scan with 128 queries per wave (eight-wave workgroups,
    // tiles of 1024 queries) measured 9 to 15 % faster than the 64-queries-per-wave tile of the
    // kernel above on large batches (4M x 256, 10 000 queries, k = 100: 11.2 -> 9.6 ms), half of that
    // with four waves, and slower on partly filled tiles (256 queries: 0.13 -> 0.17 ms): taken when
    // the padding of the batch to its tiles does not eat the gain.
    if (d_pad == 192 || d_pad == 256)
        return nq > 1024 && round_up(nq, 1024) * 87 <= round_up(nq, 256) * 100;
    return long_shape_ok(d_pad);
}

int mfma_long_wave_queries(int d_pad) { return d_pad <= 256 ? 128 : (d_pad <= 512 ? 64 : 32); }

int mfma_long_stage_rows(int d_pad, int64_t nq) { return (mfma_long_waves(d_pad, nq) == 8 && d_pad > 256) ? 64 : 32; }

// Eight waves per workgroup (one workgroup per CU, a ring of five or six stages) for large batches:
// half the corpus bytes per contraction go through the L2, measured 4 to 14 % faster at 10 000
// queries; four waves (two workgroups per CU) finish small batches sooner (16 queries on
// 500K x 1024: 0.18 against 0.22 ms).
// (rows of 1536 bytes: four waves always - 192 registers of query fragments leave no room for the
// second row block's accumulators)
int mfma_long_waves(int d_pad, int64_t nq) { return (d_pad <= 256 || (nq > 512 && d_pad <= 1024)) ? 8 : 4; }

// Collecting mode: 128 queries per wave when the rows are short enough for the registers to hold them.
// (Not for 513 to 768 queries: three tiles of 256 - register lists up to k = 10, the collecting scan
// with 64 queries per wave beyond - are a quarter less padded work than two tiles of 512, measured 4
// to 13 % faster; from 1025 queries on the wider tile's efficiency makes up for its padding.)
bool mfma_collect_wide(int64_t nq, int d_pad)
{
    return !mfma_row_split(nq, d_pad) && d_pad <= 128 && nq > 256 && !(nq > 512 && nq <= 768);
}

// Few queries: the waves of a workgroup share them and split the rows instead.
bool mfma_row_split(int64_t nq, int d_pad, bool packed) { (void)packed; return nq <= 64 && d_pad <= 256; }

int mfma_row_split_waves(int d_pad, bool packed) { return (packed ? d_pad / 2 : d_pad) <= 128 ? 4 : 2; }

bool mfma_reg_supported(int d_pad, int k) { return shape_ok(d_pad) && k >= 1 && k <= 16; }

// (any k the interface takes: about 4.6 k candidates per query survive a sample of a quarter of
// the corpus, 2.8 k a sample of half of it - taken beyond k = 512 - and the selection sorts up to 4096)
bool mfma_collect_supported(int d_pad, int k) { return (shape_ok(d_pad) || long_shape_ok(d_pad)) && k >= 1 && k <= 1024; }

bool mfma_supported(int d_pad, int k) { return mfma_reg_supported(d_pad, k) || mfma_lds_supported(d_pad, k); }

hipError_t launch_search_mfma(const SearchArgs &a, int64_t row0, int64_t row1, int S, const cand_t *seeds,
                              cand_t *lists, hipStream_t st)
{
    if (mfma_reg_supported(a.d_pad, a.k)) {
        MfmaIo o = {};
        o.seeds = seeds; o.lists = lists;
        return launch_any(a, row0, row1, S, o, st);
    }
    return launch_search_mfma_lds(a, row0, row1, S, seeds, lists, st);
}

hipError_t launch_collect_mfma(const SearchArgs &a, int64_t row0, int64_t row1, int S, const cand_t *seeds,
                               cand_t *cbuf, int32_t *ccnt, int Cs, hipStream_t st)
{
    if (!mfma_collect_supported(a.d_pad, a.k) || !seeds || !cbuf || !ccnt || Cs < 1) return hipErrorInvalidValue;
    MfmaIo o = {};
    o.seeds = seeds; o.cbuf = cbuf; o.ccnt = ccnt; o.Cs = Cs;
    return launch_any(a, row0, row1, S, o, st);
}

int mfma_collect_regions(int S, int rs_waves) { return S * (rs_waves ? rs_waves : 1); }

int mfma_seed_groups(int S, int SEG, int rs_waves) { return S * SEG * (rs_waves ? 2 * rs_waves : 2); }

int mfma_seed_segments(int S, int k, int rs_waves)
{
    const int per = rs_waves ? 2 * rs_waves : 2;   // groups a split contributes per segment
    int seg = (int)ceil_div(6 * k, per * S);   // >= 6k groups: the k-th largest is then close to
    if (seg < 1) seg = 1;                      // the k-th best item of the seeded rows
    const int most = k > 512 ? 4096 : 2048;    // (k beyond 512: with 2048 groups or fewer the k-th largest
    while (per * S * seg > most && seg > 1) --seg;   // maximum sits far below the k-th best sampled item)
    return seg;
}

// With stage_stride > 0 the seeding pass is a systematic sample: it reads one stage (64 rows, 128
// in row-split launches) every stage_stride rows, stages_per_split of them per split, so a corpus
// stored in some order (by cluster, by norm) is sampled evenly.  stage_stride = 0: rows [row0, row1).
hipError_t launch_seed_mfma(const SearchArgs &a, int64_t row0, int64_t row1, int S, int SEG, int32_t *gmax,
                            hipStream_t st, int64_t stage_stride, int stages_per_split, int64_t piece_stride,
                            int piece_stages)
{
    if (!mfma_collect_supported(a.d_pad, a.k) || !gmax) return hipErrorInvalidValue;
    MfmaIo o = {};
    o.gmax = gmax; o.SEG = SEG;
    if (piece_stride) {
        // every piece lies inside [row0, row1): the last one starts at (S * 8 * piece_stages - 1) * piece_stride
        if (a.rsplit || takes_long_scan(a) || row0 != 0 || piece_stages < 1 || piece_stride < 8 ||
            ((int64_t)S * 8 * piece_stages - 1) * piece_stride + 8 > row1)
            return hipErrorInvalidValue;
        o.piece_stride = piece_stride;
        o.piece_stages = piece_stages;
    } else if (stage_stride) {
        const int rs_rows = a.rsplit ? 32 * a.rs_waves : (takes_long_scan(a) ? mfma_long_stage_rows(a.d_pad, a.nq) : 64);
        if (stages_per_split < 1 || stage_stride < rs_rows || stage_stride % 128) return hipErrorInvalidValue;
        o.stage_stride = stage_stride;
        o.split_stride = stage_stride * stages_per_split;
        o.split_stride_rows = (int64_t)rs_rows * stages_per_split;
    }
    return launch_any(a, row0, row1, S, o, st);
}

hipError_t launch_seed_finalize(const int32_t *gmax, int64_t nq, int G, int k, cand_t *seeds, hipStream_t st,
                                int32_t *zero_word)
{
    if (nq <= 0) return hipSuccess;
    if (G > 4096) return hipErrorInvalidValue;
    const unsigned blocks = (unsigned)ceil_div(nq, (int64_t)4);
    if (G <= 256) seed_finalize_kernel<4><<<blocks, 256, 0, st>>>(gmax, nq, G, k, seeds, zero_word);
    else if (G <= 512) seed_finalize_kernel<8><<<blocks, 256, 0, st>>>(gmax, nq, G, k, seeds, zero_word);
    else if (G <= 1024) seed_finalize_kernel<16><<<blocks, 256, 0, st>>>(gmax, nq, G, k, seeds, zero_word);
    else if (G <= 2048) seed_finalize_kernel<32><<<blocks, 256, 0, st>>>(gmax, nq, G, k, seeds, zero_word);
    else seed_finalize_kernel<64><<<blocks, 256, 0, st>>>(gmax, nq, G, k, seeds, zero_word);
    return hipGetLastError();
}

}  // namespace lpq
