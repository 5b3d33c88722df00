/*
 * lpq.h - low-precision (int8) brute-force k-nearest-neighbour search on one
 * AMD Instinct MI355X (gfx950).  C ABI of liblpq.so.
 *
 * The library implements the exhaustive-search hot path of "Low-Precision
 * Quantization for Efficient Nearest Neighbor Search": a feature-wise clamped linear
 * quantizer learned from the corpus (Section 3.2, Equation 1; Sections 4.1, 4.2)
 * maps items and queries into a low-precision integer domain, the distance function
 * is evaluated on the integers (phi : Z^d x Z^d -> Z, Section 3.1), and the k nearest
 * items of every query are returned (problem statement, Section 1).
 *
 * General conventions
 *   - "dev" pointers are DEVICE pointers of the current HIP device, owned by the
 *     caller (e.g. storage of a torch tensor); "host" pointers are host memory.
 *     Matrices are row-major; `ld` is the row stride in ELEMENTS (ld >= d).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *     only enqueue work on it and do not synchronise unless stated otherwise.
 *   - Every function returning int returns LPQ_OK (0) or an error code below; on
 *     error no output buffer has been written by the failing call and
 *     lpq_last_error() describes the failure.  No C++ exception crosses the ABI.
 *   - The library owns only its two opaque handle types.  A handle may be used from
 *     one thread at a time.
 *   - Item ids are 0-based row numbers in the order the items were added.
 */
#ifndef LPQ_H
#define LPQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lpq_quantizer lpq_quantizer;
typedef struct lpq_index lpq_index;

enum {
    LPQ_OK = 0,
    LPQ_EINVAL = 1,     /* null pointer, d < 1, bits outside 1..8, ld < d, k < 1, unknown enum */
    LPQ_ERANGE = 2,     /* k > n, n >= 2^31, d beyond the int32 bound, capacity or workspace too small */
    LPQ_ENOMEM = 3,     /* device or host allocation failed */
    LPQ_EDEVICE = 4,    /* a HIP call failed */
    LPQ_ENONFINITE = 5, /* calibration data held a NaN or an infinity */
    LPQ_ESTATE = 6      /* encode before calibrate/set_params, search on an empty index */
};

/* How the range [S_b, S_e] and the offset k of Equation 1 are learned.
 *   MINMAX  S_b = min, S_e = max, k = (min + max) / 2: the observed range (Section 1,
 *           the value range the data actually occupies).
 *   ABSMAX  S_b = -A, S_e = +A, k = 0 with A the absolute maximum observed in the
 *           dimension (Section 4.2).
 *   GAUSS   S_b = mu - c sigma, S_e = mu + c sigma, k = mu, with the maximum-likelihood
 *           (1/n) estimates of a normal law per dimension; the paper uses c = 1
 *           (Section 3.2).
 *   QUANTILE  the observed range with outliers discarded (Section 4.2 leaves the technique
 *           open; here a two-sided quantile clip): of the values of the dimension sorted
 *           ascending, S_b is the one of rank floor(p (n-1)) and S_e the one of rank
 *           ceil((1-p)(n-1)) (ranks from 0), k = (S_b + S_e) / 2; p = 0 is MINMAX.  Exact
 *           order statistics (radix selection), not estimates. */
enum { LPQ_CALIB_MINMAX = 0, LPQ_CALIB_ABSMAX = 1, LPQ_CALIB_GAUSS = 2, LPQ_CALIB_QUANTILE = 3 };

/* PER_FEATURE: constants per dimension (the superscripts i of Equation 1).
 * GLOBAL: one set of constants from all n*d values, for all dimensions (Section 4.1).
 * SHARED_WIDTH: an offset per dimension and one scale for all of them - a reading of the end of
 *   Section 3.2, which asks for extra per-dimension constants (scale as well as offset) when the
 *   dimensions differ much.  The PER_FEATURE constants are learned first; then every range keeps its centre
 *   (S_b + S_e) / 2 and takes the half-width of the widest range, H = max_i (S_e - S_b) / 2
 *   (binary64 on the binary32 constants): S_b = fl32(centre - H), S_e = fl32(centre + H),
 *   k unchanged.  One code step then has the same length in every dimension, so L2SQ on codes
 *   weighs all dimensions alike (PER_FEATURE turns it into a weighted distance) while offsets
 *   between dimensions cost no code range (as they do under GLOBAL). */
enum { LPQ_SCOPE_PER_FEATURE = 0, LPQ_SCOPE_GLOBAL = 1, LPQ_SCOPE_SHARED_WIDTH = 2 };

/* L2SQ: sum_i (a_i - b_i)^2 on codes, smaller = nearer.
 * IP:   sum_i a_i b_i on codes, LARGER = nearer (maximum inner product search, Section
 *       3.1).  Angular search = IP on vectors the caller normalised to unit length. */
enum { LPQ_METRIC_L2SQ = 0, LPQ_METRIC_IP = 1 };

/* ------------------------------------------------------------------ quantizer ---- */

/* New quantizer for d-dimensional vectors and bit-width B = bits (1..8); codes lie in
 * [-2^(B-1), 2^(B-1)] and are stored one per int8 (at B = 8 the value +128 of the upper
 * clamp is stored as 127).  *out is written on success only. */
int lpq_quantizer_create(lpq_quantizer **out, int d, int bits);
void lpq_quantizer_destroy(lpq_quantizer *q);

/* Learn the constants from n >= 1 vectors x_dev[n][ld] (fp32, device).  sigma_mult is c
 * above (GAUSS; must be > 0) or the clipped fraction p per side (QUANTILE; 0 <= p < 0.5).
 * Statistics are exact for MINMAX/ABSMAX/QUANTILE; GAUSS sums in
 * fp64 (two passes: mean, then centred second moment).  This call SYNCHRONISES `stream`
 * before returning, because its status depends on the data: LPQ_ENONFINITE if a NaN or
 * an infinity was seen (the quantizer then keeps its previous state). */
int lpq_quantizer_calibrate(lpq_quantizer *q, const float *x_dev, int64_t n, int64_t ld,
                            int mode, int scope, float sigma_mult, void *stream);

/* Set / read the constants directly (host arrays of d floats each; `m` may be NULL).
 * m_i = fl32(2^B / (S_e_i - S_b_i)) is derived in fp64; a feature with S_e <= S_b gets
 * m = 0 and encodes to 0 everywhere.  Both calls synchronise the device. */
int lpq_quantizer_set_params(lpq_quantizer *q, const float *k, const float *s_b, const float *s_e);
int lpq_quantizer_get_params(const lpq_quantizer *q, float *k, float *s_b, float *s_e, float *m);

/* Equation 1 on n vectors: codes_dev[j][i] for i < d (row stride ld_codes >= d bytes;
 * bytes i >= d of a row are not touched), and, if norms_dev is not NULL, norms_dev[j] =
 * sum_i code^2 (int32).  Per value, in IEEE binary32 without fused multiply-add:
 * NaN -> 0; x < S_b -> -2^(B-1); x > S_e -> +2^(B-1); otherwise floor((x - k) * m). */
int lpq_encode(const lpq_quantizer *q, const float *x_dev, int64_t n, int64_t ld,
               int8_t *codes_dev, int64_t ld_codes, int32_t *norms_dev, void *stream);

/* ---------------------------------------------------------------------- index ---- */

/* Flat index for up to `capacity` items (1 <= capacity < 2^31).  The index takes a copy
 * of the quantizer's constants (later changes to q do not affect it) and allocates, with
 * hipMalloc, the int8 codes (rows zero padded to 64, 96, 128, 192, 256, 384, 512, 768, 1024 or
 * 1536 bytes, beyond 1536 features to a multiple of 32 bytes) and the integer norms.
 * d <= 32 768 keeps every integer distance inside int32. */
int lpq_index_create(lpq_index **out, const lpq_quantizer *q, int64_t capacity);

/* The same index with two codes per byte, for quantizers of B <= 4 bits (the memory saving
 * that Section 1 names as the first gain of a compact representation, taken below one byte per
 * feature; Section 3.1 asks for the lowest precision that keeps relative positions):
 * code c is stored as the nibble c + 8, feature 2j in the low and 2j + 1 in the high half
 * of byte j, rows padded with code 0 to 64, 96, 128, 192 or 256 features.  A nibble holds
 * -8 .. 7, so at B = 4 the top code +8 is stored as 7, for items and for queries alike (the
 * way +128 becomes 127 at B = 8); distances and norms are those of the stored codes.
 * Searches (lpq_search, lpq_search_i8) unpack in registers and give bit-identical results to
 * an unpacked index holding the same saturated codes; they take k <= 128.  Up to 128 queries run
 * the scan once per 64 queries (the small batches whose time is the corpus read: half the bytes);
 * larger batches take one scan over all queries at about the speed of an unpacked index.
 * lpq_index_data returns the packed rows (*ld_codes = bytes per row); lpq_gather_dist_i8
 * saturates the query codes the same way.  LPQ_EINVAL: B > 4; LPQ_ERANGE: d > 256. */
int lpq_index_create_packed(lpq_index **out, const lpq_quantizer *q, int64_t capacity);
void lpq_index_destroy(lpq_index *idx);

/* Append n items: fp32 vectors (encoded with the index's quantizer, Equation 1) or codes
 * produced earlier by lpq_encode with the same constants (row stride ld bytes).  Item ids are
 * the positions in add order.  Results never depend on the order of the items, but large-batch
 * search time does when near neighbours sit in adjacent rows (a corpus stored cluster by cluster:
 * up to ~2x slower, see lpq_search_overflow_stats); adding the items in shuffled order avoids it. */
int lpq_index_add_f32(lpq_index *idx, const float *x_dev, int64_t n, int64_t ld, void *stream);
int lpq_index_add_i8(lpq_index *idx, const int8_t *codes_dev, int64_t n, int64_t ld, void *stream);
int64_t lpq_index_size(const lpq_index *idx);  /* items added so far; -1 for NULL */

/* Read-only view of the index storage (device pointers owned by the index, valid until it
 * is destroyed): codes [size][*ld_codes] int8 and norms [size] int32.  Any may be NULL. */
int lpq_index_data(const lpq_index *idx, const int8_t **codes_dev, int64_t *ld_codes,
                   const int32_t **norms_dev);

/* --------------------------------------------------------------------- search ---- */

/* Bytes of device workspace lpq_search / lpq_search_i8 need for nq queries and k results
 * (0 on invalid arguments).  The workspace needs 256-byte alignment. */
size_t lpq_search_workspace_bytes(const lpq_index *idx, int64_t nq, int k, int metric);

/* k nearest items of each of nq queries q_dev[nq][ld] (fp32; encoded with the index's
 * quantizer exactly like the items).  Outputs, row i = query i, best first:
 *   ids_dev [nq][k] int32 item ids;
 *   dist_dev[nq][k] int32: L2SQ the full integer distance sum (cq - cx)^2, ascending;
 *                          IP the integer inner product, descending.
 * Equal distances are ordered by ascending id, so the result is unique.
 * 1 <= k <= min(size, 1024).  nq = 0 is a no-op.  Asynchronous on `stream`.
 * Every shape returns the same exact result; speed differs: indexes of up to 1536 features are
 * searched on the matrix cores for every k and batch size once they hold enough items for a
 * threshold sample (a few ten thousand), longer vectors and smaller indexes by a plain
 * dot-product kernel (about two orders of magnitude slower per contraction). */
int lpq_search(const lpq_index *idx, const float *q_dev, int64_t nq, int64_t ld, int k,
               int metric, int32_t *ids_dev, int32_t *dist_dev, void *workspace_dev,
               size_t workspace_bytes, void *stream);

/* lpq_search for callers that cannot allocate device memory or pass a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and errors as lpq_search, but the intermediates (query codes, group maxima, candidate lists or
 * regions, counters) live in a device array that is part of the library: LPQ_STATIC_WORKSPACE_BYTES
 * on every GPU the library is used on, held until the process ends.  The call allocates nothing
 * (no hipMalloc / hipFree, no allocating library routine) and is kernel launches only, after one
 * hipGetSymbolAddress per device on the first call there.  A search whose plan needs more than
 * LPQ_STATIC_WORKSPACE_BYTES (lpq_search_workspace_bytes tells) returns LPQ_ERANGE and launches
 * nothing: the limit is meant for small batches (e.g. 1M x 128: up to 256 queries at k = 10, 48 at
 * k = 100).  All calls on one GPU share the array, which keeps the previous call's contents (every
 * counter in it is cleared by the kernels that precede its use): calls that overlap on one GPU -
 * different streams, or different threads - race; serialise them on one stream. */
#define LPQ_STATIC_WORKSPACE_BYTES (64u << 20)
int lpq_search_static(const lpq_index *idx, const float *q_dev, int64_t nq, int64_t ld, int k,
                      int metric, int32_t *ids_dev, int32_t *dist_dev, void *stream);

/* Same, for queries that are already codes (int8, row stride ld bytes). */
int lpq_search_i8(const lpq_index *idx, const int8_t *qcodes_dev, int64_t nq, int64_t ld, int k,
                  int metric, int32_t *ids_dev, int32_t *dist_dev, void *workspace_dev,
                  size_t workspace_bytes, void *stream);

/* Exact search on the original fp32 vectors (the reference set S_E of the recall
 * definition, Section 5.3): x_dev[n][ldx], q_dev[nq][ldq], fp32 arithmetic (the squared
 * distance is summed directly as (q - x)^2, never through norms).  dist_dev [nq][k] fp32,
 * L2SQ ascending / IP descending, ties to the lower id.  1 <= k <= min(n, 1024).  A workgroup keeps
 * a query vector and its candidate buffer in 64 KB of LDS, which bounds d: at most 15 328 features
 * for k <= 256, 12 256 for k = 1024 (in between: (65 408 - 8 c) / 4 rounded down to a multiple of 4,
 * c = the power of two >= max(2 k, k + 256)); beyond that LPQ_ERANGE, and the workspace query
 * returns 0. */
size_t lpq_search_f32_workspace_bytes(int64_t n, int64_t nq, int d, int k);
int lpq_search_f32(const float *x_dev, int64_t n, int64_t ldx, const float *q_dev, int64_t nq,
                   int64_t ldq, int d, int k, int metric, int32_t *ids_dev, float *dist_dev,
                   void *workspace_dev, size_t workspace_bytes, void *stream);

/* ------------------------------------------------------------ candidate lists ---- */

/* Integer distances between each query and the items its id list names: the distance
 * routine that Section 5.2 swaps into graph indexes, phi(Q(q), Q(x_id)), as one batched
 * call.  qcodes_dev int8 [nq][ld] are codes of the index's quantizer (lpq_encode), ld >= d;
 * ids_dev int32 [nq][m]; dist_dev int32 [nq][m] receives sum (cq - cx)^2 (L2SQ) or
 * sum cq cx (IP).  An id outside [0, size) means "no item" and gives INT32_MAX (L2SQ) /
 * INT32_MIN (IP).  On a packed index the distances are those of the stored (saturated) codes
 * and of the query codes saturated to -8 .. 7.  All buffers are the caller's device memory;
 * asynchronous on stream.
 * LPQ_EINVAL: null argument, m < 1, ld < d, unknown metric; LPQ_ESTATE: empty index. */
int lpq_gather_dist_i8(const lpq_index *idx, const int8_t *qcodes_dev, int64_t nq, int64_t ld,
                       const int32_t *ids_dev, int m, int metric, int32_t *dist_dev, void *stream);

/* Second stage on the original vectors, recovering the recall that quantization costs
 * (the 2-6 % of Section 5.3): for each query the exact distance (binary64 sums) to each of
 * its kc candidates cand_ids_dev [nq][kc] (e.g. the ids of an int8 search with k' > k),
 * the k best sorted by (distance, id): ids_dev int32 [nq][k], dist_dev fp32 [nq][k]
 * (L2SQ ascending / IP descending).  Candidate ids outside [0, n) are skipped; if fewer
 * than k remain the row is completed with id -1 and distance +inf (L2SQ) / -inf (IP).
 * 1 <= kc <= 4096, k >= 1.  Asynchronous on stream; no workspace.
 * LPQ_EINVAL: null argument, d < 1, ldx/ldq < d, kc or k < 1, unknown metric; LPQ_ERANGE:
 * kc > 4096. */
int lpq_rerank_f32(const float *x_dev, int64_t n, int64_t ldx, const float *q_dev, int64_t nq,
                   int64_t ldq, int d, const int32_t *cand_ids_dev, int kc, int k, int metric,
                   int32_t *ids_dev, float *dist_dev, void *stream);

/* ---------------------------------------------------------------- diagnostics ---- */

/* Process-wide tuning knobs for measurements; 0 restores the built-in choice.
 *   LPQ_TUNE_PATH        1 = generic dot-product kernel, 2 = matrix-core kernels (built-in
 *                        choice of variant), 3 = the collecting matrix-core variant for every
 *                        k it takes, 4 = matrix-core kernels without the
 *                        collecting variant
 *   LPQ_TUNE_SPLITS      number of corpus splits per query tile in the main pass
 *   LPQ_TUNE_SEED_ROWS   rows of the threshold-seeding pass (0 = built-in choice,
 *                        -1 = no seeding pass)
 *   LPQ_TUNE_DRY_RUN     timing ablations of the matrix-core kernel whose results are meaningless
 *                        (1 never collects a candidate, 2 no workgroup barrier, 3 no corpus
 *                        copies, 4 neither, 5 candidates detected but not queued, 6 queued but
 *                        not processed, 7 every copy reads the first two stages of its split, which
 *                        stay in L2).  Compiled only into builds made with -DLPQ_ABLATION
 *                        (python -m paper_2110_08919_amd.build --ablation writes
 *                        liblpq_ablation.so); the shipped library has none of these branches
 *                        and rejects a non-zero value with LPQ_EINVAL.
 *   LPQ_TUNE_WORK_ORDER  how workgroups of the matrix-core kernel are dealt to (split, query tile)
 *                        pairs: 0 built-in, 1 each XCD takes whole splits, 2 each XCD takes whole
 *                        query tiles, 3 plain block order
 *   LPQ_TUNE_WAVE_QUERIES queries per wave of the collecting variant: 64 or 128 (0 = built-in)
 *   LPQ_TUNE_REGION_CAP  candidates a region of the collecting variant holds (0 = built-in); a tiny
 *                        value makes most queries overflow and go through the exact redo paths
 * Results never depend on PATH, SPLITS, SEED_ROWS, WORK_ORDER, WAVE_QUERIES or REGION_CAP.
 * The knobs are atomics: setting one while other threads search is not a data race; a search
 * reads each knob at some moment of its planning, so set them before the searches they are for
 * (lpq_search_workspace_bytes and the lpq_search that uses its answer must see the same values). */
enum { LPQ_TUNE_PATH = 0, LPQ_TUNE_SPLITS = 1, LPQ_TUNE_SEED_ROWS = 2, LPQ_TUNE_DRY_RUN = 3, LPQ_TUNE_WORK_ORDER = 4,
       LPQ_TUNE_WAVE_QUERIES = 5, LPQ_TUNE_REGION_CAP = 6, LPQ_TUNE_COUNT_ = 7 };
int lpq_set_tuning(int key, int64_t value);

/* Kernel timing for benchmarks.  While enabled, every launch of the contraction/top-k
 * kernel of lpq_search* (LPQ_PROFILE_SCAN) and of its threshold-seeding pass
 * (LPQ_PROFILE_SEED) is bracketed by a pair of HIP events on the launch stream.
 * lpq_profile_read synchronises those events and returns the number of bracketed
 * launches and their summed duration in milliseconds since the last enable;
 * lpq_profile_read_kind does the same for one kind of launch. */
enum { LPQ_PROFILE_SCAN = 0, LPQ_PROFILE_SEED = 1 };
int lpq_profile_enable(int on);
int lpq_profile_read(int64_t *launches, double *total_ms);
int lpq_profile_read_kind(int kind, int64_t *launches, double *total_ms);

/* How lpq_search would run a search, computed on the host without any device or index: the plan
 * for nq queries and k results on an index of n_items items of d features at `bits` bits (packed:
 * two codes per byte).  For capacity planning (out[16] is what lpq_search_workspace_bytes would
 * return less its 256 bytes of alignment slack) and for checking the planner itself.  out receives
 * LPQ_PLAN_INFO_COUNT values:
 *   [0] kernel family (0 generic dot-product kernel, 1 matrix-core with lists in LDS, 2 matrix-core
 *       with lists in registers, 3 matrix-core collecting scan)   [1] row-split workgroups (0/1)
 *   [2] waves of a row-split workgroup   [3] queries per wave of the collecting scan
 *   [4] query rows the workspace holds (padded)   [5] rows of the threshold-seeding pass (0 = none)
 *   [6] corpus splits of the seeding pass   [7] corpus splits of the main scan   [8] segments per split
 *   and [9] group maxima per query of the seeding pass   [10] candidate regions per query and
 *   [11] their capacity (collecting scan)   [12] splits of the generic redo   [13] splits of the
 *   register-list redo   [14] further rounds of the collecting scan   [15] lists merged per workgroup
 *   in a first merge pass (0 = one pass)   [16] workspace bytes   [17] offset of the per-tile plan
 *   inside the workspace (packed index; else 0)
 *   [18..33] byte offsets of the plan's buffers in the order they are laid out (0 = not used), [34]
 *   their end.  Every offset is a multiple of 256 and the used ones never decrease.  (A packed
 *   index is searched in tiles of 64 queries unless one collecting scan takes the whole batch: the
 *   values then describe the plan of a full tile, [4], [16] and [17] the whole workspace.)
 * LPQ_EINVAL / LPQ_ERANGE as for lpq_quantizer_create, lpq_index_create and lpq_search. */
#define LPQ_PLAN_INFO_COUNT 35
int lpq_search_plan_info(int d, int bits, int packed, int64_t n_items, int64_t nq, int k, int64_t *out,
                         int out_count);

/* Attainable-rate probes (benchmarks only): what this GPU sustains on the two resources that
 * bound lpq_search, measured by kernels that do nothing else, so that a roofline fraction quoted
 * against a published peak can be read next to what the part reaches in practice.  Both calls
 * allocate a small device buffer, time with events on `stream` and synchronise it.
 *   lpq_probe_mfma_i8: a register-resident loop of the int8 matrix instruction the search uses
 *     (the contraction of Section 3.1's phi on codes), `iters` x 8 instructions per wave, four
 *     waves per workgroup, two workgroups per CU.  The operand registers are filled from
 *     operands_dev[operand_bytes] (device memory, 16-byte aligned; null = all-zero operands): the
 *     sustained rate depends on how many operand bits toggle, so pass the bytes of interest
 *     (random bytes, or the codes of an index).  *tops = 1e12 integer operations per second.
 *   lpq_probe_scan_core: the inner loop of the batched scan and nothing else - per 32 rows and 128
 *     queries of a wave sixteen matrix instructions with the filter epilogue (maximum of the 16
 *     accumulators of a lane, threshold compare, branch) and the row operands and accumulator seeds
 *     read from LDS - without corpus copies, barriers or candidates; `stages` x 64 instructions
 *     per wave.  LDS ring and query registers are filled from operands_dev as above.  *tops as
 *     above: the ceiling of that loop on this GPU for such operand bits.
 *   lpq_probe_stream: reads bytes (rounded down to a multiple of 4096) of src_dev `reps` times,
 *     mode 0 through the asynchronous global->LDS copies of the scan kernels, mode 1 through
 *     16-byte register loads.  *gbps = 1e9 bytes per second.
 * LPQ_EINVAL: null output, iters or stages outside 1..10 000 000, misaligned or too small a buffer,
 * unknown mode, reps outside 1..10 000. */
int lpq_probe_mfma_i8(const void *operands_dev, size_t operand_bytes, int iters, double *tops, void *stream);
int lpq_probe_scan_core(const void *operands_dev, size_t operand_bytes, int stages, double *tops, void *stream);
int lpq_probe_stream(const void *src_dev, size_t bytes, int mode, int reps, double *gbps, void *stream);

/* Diagnostics of the collecting variant: after a search with the same (idx, nq, k, metric) and
 * workspace has finished, the number of queries whose candidates did not fit and that were
 * searched again (up to 64 by the generic kernel, more by a pass of the register-list
 * matrix-core kernel when k <= 16; 0 when the search did not use the collecting variant) and the
 * largest number of candidates any region received in the last round of the scan.  Synchronises
 * the device. */
int lpq_search_overflow_stats(const lpq_index *idx, int64_t nq, int k, int metric, const void *workspace_dev,
                              int64_t *redone_queries, int64_t *max_region_fill);

/* For k > 16 more than 16 such queries are not searched again exactly at once: the scan
 * runs again (up to two more rounds) over the query tiles that hold one, with bounds taken from
 * the candidates the round before did collect, and only queries that overflow every time go
 * through the generic kernel.  *left_queries = their number after the last search (0 when the
 * plan has no further rounds or they did not run).  Same arguments and synchronisation as above. */
int lpq_search_overflow_left(const lpq_index *idx, int64_t nq, int k, int metric, const void *workspace_dev,
                             int64_t *left_queries);

/* Message of the last error on the calling thread ("" if none). */
const char *lpq_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* LPQ_H */
