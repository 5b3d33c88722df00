// Internal declarations shared by the translation units of liblpq.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "lpq.h"

namespace lpq {

// ---------------------------------------------------------------------------------
// Candidate keys.  Inside the search every (item, query) pair is ranked by the pair
//   key = nx_j - 2 * dot(cq_i, cx_j)      (nx_j = sum of squared codes of item j; 0 for IP)
// which differs from the squared distance only by the per-query constant |cq_i|^2 and
// from the inner product by the factor -2, so "smaller key = nearer" for both metrics.
// A candidate is the 64-bit word  (key biased to unsigned) << 32 | id : one unsigned
// compare orders by (key ascending, id ascending), the tie rule of the interface.
// ---------------------------------------------------------------------------------
typedef unsigned long long cand_t;
static const cand_t CAND_NONE = ~0ull;  // sorts after every real candidate

__host__ __device__ inline cand_t make_cand(int32_t key, uint32_t id)
{
    return ((cand_t)((uint32_t)key ^ 0x80000000u) << 32) | (cand_t)id;
}
__host__ __device__ inline int32_t cand_key(cand_t c) { return (int32_t)((uint32_t)(c >> 32) ^ 0x80000000u); }
__host__ __device__ inline uint32_t cand_id(cand_t c) { return (uint32_t)c; }

// Ranking modes of the merge kernel: the two integer metrics (same values as the public
// LPQ_METRIC_* constants) and the two fp32 ones, whose keys are order-preserving integer
// images of the float distance (L2) or of minus the inner product (IP).
enum { MODE_I8_L2 = 0, MODE_I8_IP = 1, MODE_F32_L2 = 2, MODE_F32_IP = 3,
       MODE_I8_IP_ADJ = 4 };   // inner product plus a per-query term (packed corpus codes are stored + 8)

// Order-preserving map between finite floats and int32 (its own inverse); -0 is folded into +0.
__host__ __device__ inline int32_t float_to_sortable(float f)
{
    f += 0.0f;
    int32_t b;
    __builtin_memcpy(&b, &f, 4);
    return b >= 0 ? b : (b ^ 0x7fffffff);
}
__host__ __device__ inline float sortable_to_float(int32_t s)
{
    const int32_t b = s >= 0 ? s : (s ^ 0x7fffffff);
    float f;
    __builtin_memcpy(&f, &b, 4);
    return f;
}

__host__ __device__ static inline int next_pow2(int v)
{
    int p = 1;
    while (p < v) p <<= 1;
    return p;
}
static inline int64_t round_up(int64_t v, int64_t m) { return (v + m - 1) / m * m; }
static inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }

enum { MAX_K = 1024, MAX_D = 32768, MAX_K_PACKED = 128, MAX_D_PACKED = 256 };

// Per-feature constants on the device: four arrays of d floats, [k | S_b | S_e | m].
struct QuantParams {
    const float *k, *sb, *se, *m;
    int d, bits;
};

// ---- quantizer kernels (quant_kernels.hip) ---------------------------------------
// Calibration scratch layout is private to quant_kernels.hip; the API allocates
// calib_scratch_bytes(d) bytes once per quantizer.
size_t calib_scratch_bytes(int d);
hipError_t launch_calibrate(const float *x, int64_t n, int64_t ld, int d, int bits, int mode,
                            int scope, double sigma_mult, void *scratch, float *params_out,
                            int *nonfinite_flag, hipStream_t st);
hipError_t launch_derive_m(float *params, int d, int bits, hipStream_t st);
// Equation 1 on n rows.  zero_pad_to > d additionally writes zero bytes for columns
// d .. zero_pad_to-1 of each row; n_out > n additionally writes rows n .. n_out-1 as zero codes
// (and zero norms).
hipError_t launch_encode(const QuantParams &qp, const float *x, int64_t n, int64_t ld, int8_t *codes,
                         int64_t ldc, int zero_pad_to, int32_t *norms, hipStream_t st, int64_t n_out = 0);
// Copy codes into padded rows (zero padding), computing norms.
hipError_t launch_repack_i8(const int8_t *src, int64_t n, int64_t ld, int d, int8_t *dst, int64_t ldd,
                            int d_pad, int32_t *norms, hipStream_t st, int64_t n_out = 0);
// Derived per-item arrays used by the matrix-core kernel: cinit_j = -ceil(nx_j / 2) and one
// word of 32 parity bits (bit r = nx_{32w+r} & 1) per 32 items; rows >= n of the last word's
// block get cinit = CINIT_PAD.  use_norms = false (IP) gives cinit = 0 and parity = 0.
hipError_t launch_zero_bytes(void *p, size_t bytes, hipStream_t st);
// Sub-byte packing: int8 codes [n][ld] -> two codes per byte (stored + 8, clamped to [-8, 7]),
// rows of d_pad / 2 bytes, and the norms of the stored codes.
hipError_t launch_pack4(const int8_t *src, int64_t n, int64_t ld, int d, uint8_t *dst, int d_pad, int32_t *norms,
                        hipStream_t st);
// Queries for the packed scan: codes permuted inside every group of 16 to match the operand
// unpacking, and qadj[q] = |cq|^2 + 16 sum(cq) (L2SQ) or -8 sum(cq) (IP).
hipError_t launch_permute_queries(const int8_t *q, int64_t nq_pad, int d_pad, bool l2, int8_t *qperm, int32_t *qadj,
                                  hipStream_t st);  // bytes % 4 == 0, p 4-byte aligned
hipError_t launch_item_aux(const int32_t *norms, int64_t row0, int64_t n_total, int32_t *cinit,
                           uint32_t *parity, hipStream_t st);

// ---- search kernels ---------------------------------------------------------------
struct SearchArgs {
    const int8_t *codes;    // [n][d_pad]
    const int32_t *norms;   // [n] (ignored for IP)
    const int32_t *cinit;   // [round_up(n,32)]
    const uint32_t *parity; // [ceil(n/32)]
    int64_t n;
    int d_pad;
    const int8_t *qcodes;   // [nq_pad][d_pad], zero padded
    int64_t nq;
    int k;
    int metric;
    bool rsplit;            // register variant: row-split workgroups (set from mfma_row_split)
    int rs_waves = 4;       // ... of this many waves (mfma_row_split_waves): a stage holds 32 rows per wave
    int dry_run = 0;        // builds with -DLPQ_ABLATION only: timing experiments whose results are meaningless
    int work_order = 0;     // matrix-core kernels: block -> (split, query tile) mapping (0 = built-in)
    int wave_queries = 64;  // collecting mode: queries per wave (64 or 128)
    bool packed = false;    // codes holds two 4-bit codes (stored + 8) per byte, rows of d_pad / 2 bytes; qcodes permuted to match
    // Redo pass of the register-list kernel (device memory written by an earlier kernel): a workgroup
    // works only if more than redo_min queries are flagged in all and one of its own queries is.
    const int32_t *redo_flags = nullptr;   // [nq] non-zero = search this query again
    const int32_t *redo_count = nullptr;   // number of flagged queries
    int redo_min = 0;
};

// Queries of the collecting scan that must be searched again: up to this many go through the
// generic kernel (a fixed grid shares them out), more through a pass of the register-list kernel
// whose workgroups skip query tiles without a flagged query.
constexpr int REDO_GENERIC_MAX = 64;

// Generic kernel: one workgroup per (query, corpus split); any d_pad (multiple of 32), any k.
// Writes lists[(q * S + s) * k + r], sorted ascending, CAND_NONE-filled.
hipError_t launch_search_generic(const SearchArgs &a, int64_t row0, int64_t row1, int S,
                                 const cand_t *seeds, cand_t *lists, hipStream_t st);
// The same for the *qcount queries listed in qlist (device memory, written by an earlier kernel):
// a fixed grid shares out the (query, split) pairs; lists of other queries are left untouched.
// Does nothing if more than max_listed queries are listed.
hipError_t launch_search_generic_list(const SearchArgs &a, int64_t row0, int64_t row1, int S, const int32_t *qlist,
                                      const int32_t *qcount, cand_t *lists, hipStream_t st, int max_listed = INT32_MAX);

// Matrix-core kernels.  search_mfma.hip keeps the k best of a query in registers (k <= 16) and
// has a seeding pass; search_mfma_lds.hip keeps them in LDS (larger k).  launch_search_mfma
// picks the variant; row0 must be a multiple of 64.
bool mfma_supported(int d_pad, int k);
bool mfma_reg_supported(int d_pad, int k);
bool mfma_lds_supported(int d_pad, int k);
hipError_t launch_search_mfma(const SearchArgs &a, int64_t row0, int64_t row1, int S, const cand_t *seeds,
                              cand_t *lists, hipStream_t st);
hipError_t launch_search_mfma_lds(const SearchArgs &a, int64_t row0, int64_t row1, int S, const cand_t *seeds,
                                  cand_t *lists, hipStream_t st);
// Seeding pass: group maxima gmax[nq_pad][G], G = mfma_seed_groups(S, SEG, rsplit), over the sampled
// rows (all of them real items), then seeds[q] = bound from the k-th largest group maximum.
int mfma_seed_segments(int S, int k, int rs_waves);   // rs_waves: waves of a row-split workgroup, 0 = not row-split
int mfma_seed_groups(int S, int SEG, int rs_waves);      // = G, entries per query in gmax
int mfma_queries_per_workgroup(int64_t nq, int d_pad, bool wide = false);   // query tile; wide: 128 queries per wave
bool mfma_collect_wide(int64_t nq, int d_pad);           // collecting mode may use 128 queries per wave
bool mfma_row_split(int64_t nq, int d_pad, bool packed = false);   // few queries: waves split rows, share queries
bool mfma_long_rows(int d_pad, int64_t nq);         // rows of 384 to 1536 bytes, and large batches on 192 and 256: their own collecting scan and seeding pass
int mfma_long_waves(int d_pad, int64_t nq);           // ... in workgroups of this many waves (4: two workgroups per CU, 8: one)
int mfma_long_stage_rows(int d_pad, int64_t nq);   // ... whose stages hold 32 or 64 rows (the unit of the seeding pass' sample)
int mfma_long_wave_queries(int d_pad);     // ... which keep 64 (up to 512 bytes) or 32 queries per wave
int mfma_row_split_waves(int d_pad, bool packed);   // 4 on rows of up to 128 bytes, 2 on longer ones (collecting scan and seeding pass only)
// With stage_stride > 0 (a multiple of 128) the pass is a systematic sample of [row0, row1): one
// stage (64 rows; 128 in row-split launches) every stage_stride rows, stages_per_split per split.
// With piece_stride > 0 instead (not for row-split launches; row0 = 0): a finer systematic sample,
// runs of 8 rows every piece_stride rows, dealt round-robin to the splits, eight runs to a stage,
// piece_stages stages per split - neighbouring rows of the corpus then fall into different groups.
hipError_t launch_seed_mfma(const SearchArgs &a, int64_t row0, int64_t row1, int S, int SEG, int32_t *gmax,
                            hipStream_t st, int64_t stage_stride = 0, int stages_per_split = 0,
                            int64_t piece_stride = 0, int piece_stages = 0);
// Collecting scan (any k up to MAX_K): thresholds stay at seeds[q] (required); every candidate beating its
// query's seed is appended to cbuf[(q * SS + region) * Cs + ...], SS = mfma_collect_regions(S, rsplit),
// and ccnt[q * SS + region] = number offered (entries beyond Cs were dropped).
bool mfma_collect_supported(int d_pad, int k);
int mfma_collect_regions(int S, int rs_waves);
hipError_t launch_collect_mfma(const SearchArgs &a, int64_t row0, int64_t row1, int S, const cand_t *seeds,
                               cand_t *cbuf, int32_t *ccnt, int Cs, hipStream_t st);
// Per query: if no region overflowed and at most 4096 candidates were collected, sort them, write
// the k best as the final result and set over[q] = 0; otherwise set over[q] = 1 and write nothing.
// expected_candidates (per query, 0 = unknown) picks the one-wave-per-query kernel when small (k <= 32,
// SS <= 64); that kernel takes any number of candidates the regions hold.
// Flagged queries are also appended to qlist[atomicAdd(qcount, 1)] (qcount must be zero before).
hipError_t launch_collect_select(const cand_t *cbuf, const int32_t *ccnt, int64_t nq, int SS, int Cs, int k,
                                 int32_t *over, int32_t *qlist, int32_t *qcount, int32_t *ids, int32_t *dists,
                                 const int32_t *qnorms, int metric, hipStream_t st, int expected_candidates = 0,
                                 const int32_t *only = nullptr,   // only (optional): int[nq]; other queries just get over[q] = 0,
                                 const int32_t *gate_count = nullptr, int gate_min = 0);   // and so do all unless *gate_count > gate_min
// Second round of the collecting scan for queries flagged by launch_collect_select: bounds_out[q] =
// the k-th best of what the first round collected for q (a bound on its final k-th best), or
// bounds_in[q] if that was fewer than k; queries not flagged, and all of them unless
// *qcount > min_flagged, get the bound that nothing passes.  zero_word (optional) is set to 0.
hipError_t launch_collect_refine(const cand_t *cbuf, const int32_t *ccnt, int64_t nq, int SS, int Cs, int k,
                                 const int32_t *over, const int32_t *qcount, int min_flagged, const cand_t *bounds_in,
                                 cand_t *bounds_out, int32_t *zero_word, hipStream_t st);
// zero_word (optional): one int the kernel also sets to 0 (the counter of the redo list).
hipError_t launch_seed_finalize(const int32_t *gmax, int64_t nq, int G, int k, cand_t *seeds, hipStream_t st,
                                int32_t *zero_word = nullptr);

// Merge P lists of k candidates per query into one (merge.hip).  If ids/dists are given the
// result is final: ids, and dist = key + qnorm (L2SQ) or -key/2 (IP).  Otherwise the merged
// candidates go to out_lists[q][k] (sorted) and, if seeds_out, seeds_out[q] = the k-th best
// candidate (CAND_NONE when fewer than k exist).  sorted_lists: every input list is in
// ascending order (allows the selection kernel for small k and many lists).
hipError_t launch_merge(const cand_t *lists, int64_t nq, int P, int k, const cand_t *extra_lists,
                        cand_t *out_lists, cand_t *seeds_out, int32_t *ids, int32_t *dists,
                        const int32_t *qnorms, int metric, hipStream_t st, bool sorted_lists = false,
                        const int32_t *only = nullptr,   // only (optional): int[nq]; queries with only[q] == 0 are skipped
                        const int32_t *gate_count = nullptr, int gate_lo = 0,   // gate (optional): nothing is done
                        int gate_hi = INT32_MAX);                               // unless gate_lo <= *gate_count <= gate_hi
int merge_max_lists(int k);
int merge_max_sorted_lists(int k);   // same for lists that are each sorted (k <= 32: more of them)
// First pass of a two-pass merge: groups of `group` consecutive lists of each query are merged
// into out_lists[q][ceil(P/group)][k].
hipError_t launch_merge_groups(const cand_t *lists, int64_t nq, int P, int group, int k, cand_t *out_lists,
                               hipStream_t st);

// ---- candidate lists (candidates.hip) -------------------------------------------------
// out[i][j] = integer distance between query i (int8 codes, stride ldq) and item ids[i][j];
// ids outside [0, n) give INT32_MAX (L2SQ) / INT32_MIN (IP).
hipError_t launch_gather_dist(const int8_t *codes, const int32_t *norms, int64_t n, int d, int d_pad, const int8_t *q,
                              int64_t nq, int64_t ldq, const int32_t *ids, int m, int metric, int32_t *out,
                              hipStream_t st, bool packed = false);   // packed: rows of d_pad / 2 bytes, two codes per byte stored + 8; queries saturate to -8 .. 7
// Exact distances (binary64 sums) of each query's kc <= 4096 candidates on the fp32 vectors, the k
// best sorted by (distance, id); ids outside [0, n) are skipped, missing results are id -1.
hipError_t launch_rerank_f32(const float *x, int64_t n, int64_t ldx, const float *q, int64_t nq, int64_t ldq, int d,
                             const int32_t *cand, int kc, int k, int metric, int32_t *ids, float *dists, hipStream_t st);

// ---- fp32 exact search (search_f32.hip) ---------------------------------------------
size_t f32_workspace_bytes(int64_t n, int64_t nq, int d, int k);
int f32_max_d(int k);   // largest d the fp32 search takes for k results (its LDS holds a query and its candidates)
hipError_t launch_search_f32(const float *x, int64_t n, int64_t ldx, const float *q, int64_t nq,
                             int64_t ldq, int d, int k, int metric, int32_t *ids, float *dists,
                             void *ws, hipStream_t st);

// ---- attainable-rate probes (probe.hip); they allocate a small sink, time with events on st and synchronise ----
// Sustained rate of a register-resident v_mfma_i32_32x32x32_i8 loop whose operand registers are
// filled from `operands` (null: all zero), in 1e12 integer operations per second.
hipError_t probe_mfma(const void *operands, size_t bytes, int iters, double *tops, hipStream_t st);
// Sustained rate of the wide collecting scan's inner loop alone (matrix instructions, filter epilogue,
// operands from an LDS ring filled once from `operands`; no copies, barrier or candidates), in 1e12 op/s.
hipError_t probe_scan_core(const void *operands, size_t bytes, int stages, double *tops, hipStream_t st);
// Sustained read rate over `bytes` of device memory, `reps` passes: mode 0 through asynchronous
// global->LDS copies into wave-private rings (bytes / 4096 chunks are read), mode 1 through
// 16-byte register loads; in 1e9 bytes per second.
hipError_t probe_stream(const void *src, size_t bytes, int mode, int reps, double *gbps, hipStream_t st);

static const int32_t CINIT_PAD = -(1 << 30);

}  // namespace lpq
