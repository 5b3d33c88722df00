/*
 * CPU oracle for low-precision (integer) brute-force k-nearest-neighbour search.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain, slow, obviously-correct
 * statement of what the search path computes, written from the paper
 * ("Low-Precision Quantization for Efficient Nearest Neighbor Search").  It is
 * used by the tests, by the smoke check and by the benchmark's CPU-baseline leg,
 * and by nothing else; it shares no code, header, table or helper with the GPU
 * library, and the GPU library never calls it.
 *
 * Every function is the definition written out: no blocking, no fusion, no
 * reordering, no intrinsics.  (The only concession to run time is an optional
 * OpenMP "parallel for" over independent queries.)
 *
 *   calibration   Section 3.2 (Gaussian maximum likelihood: S_b = mu - sigma,
 *                 S_e = mu + sigma, k = mu), Section 4.1 (one mu, sigma for all
 *                 dimensions), Section 4.2 (absolute maximum per dimension),
 *                 plus the [min, max] reading of Section 1 (the value range the
 *                 data actually occupies); and, for the closing remark of Section
 *                 3.2 (dimensions that differ much need extra per-dimension
 *                 constants, for scale as well as offset), a scope with one offset
 *                 per dimension and one range width for all of them.
 *   encode        Equation 1, evaluated in IEEE binary32 as two rounded
 *                 operations t = (x - k) * m with m = fl32(2^B / (S_e - S_b)),
 *                 then floor; the result +2^(B-1) of the upper clamp is kept for
 *                 B < 8 and saturated to 127 when stored in a byte at B = 8.
 *   distance      phi : Z^d x Z^d -> Z of Section 3.1: squared Euclidean
 *                 distance sum (a_i - b_i)^2, or the inner product sum a_i b_i
 *                 (larger = nearer; the "angular" row of Table 2 is the inner
 *                 product of codes of unit-normalised vectors).
 *   top-k         Section 1's problem statement: the k items of smallest
 *                 distance; here by sorting ALL n (distance, id) pairs, ties
 *                 going to the lower id.
 *   exact search  the S_E of Section 5.3: the same on the fp32 vectors, with the
 *                 sums accumulated in binary64.
 *   recall        |S_E intersect S_A| / |S_E| of Section 5.3.
 *   gather        phi between a query and the items of an id list (the routine
 *                 Section 5.2 replaces inside graph indexes).
 *   re-rank       exact distances of a candidate list on the fp32 vectors, sorted.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

enum { LPQO_MINMAX = 0, LPQO_ABSMAX = 1, LPQO_GAUSS = 2, LPQO_QUANTILE = 3 };
enum { LPQO_PER_FEATURE = 0, LPQO_GLOBAL = 1, LPQO_SHARED_WIDTH = 2 };
enum { LPQO_L2SQ = 0, LPQO_IP = 1 };

/* m = fl32( 2^B / (S_e - S_b) ), the multiplier of Equation 1; 0 marks a feature
 * whose range is empty (S_e <= S_b), which encodes to code 0 everywhere. */
void lpqo_derive_m(const float *sb, const float *se, int d, int bits, float *m)
{
    for (int i = 0; i < d; ++i) {
        double width = (double)se[i] - (double)sb[i];
        m[i] = (width > 0.0) ? (float)(ldexp(1.0, bits) / width) : 0.0f;
    }
}

/* Range statistics of one set of values visited through (first, count, stride
 * pattern given by the caller loop); kept as a struct to serve both scopes. */
typedef struct {
    double mn, mx, amax, sum;
    int64_t cnt;
    int bad; /* a NaN or an infinity was seen */
} stat_t;

static void stat_init(stat_t *s)
{
    s->mn = INFINITY; s->mx = -INFINITY; s->amax = 0.0; s->sum = 0.0; s->cnt = 0; s->bad = 0;
}

static void stat_add(stat_t *s, float v)
{
    if (!isfinite(v)) { s->bad = 1; return; }
    double x = (double)v;
    if (x < s->mn) s->mn = x;
    if (x > s->mx) s->mx = x;
    if (fabs(x) > s->amax) s->amax = fabs(x);
    s->sum += x;
    s->cnt += 1;
}

static void constants_from(int mode, double sigma_mult, double mn, double mx, double amax,
                           double mu, double sigma, float *k, float *sb, float *se)
{
    if (mode == LPQO_GAUSS) {          /* Section 3.2: S_b = mu - sigma, S_e = mu + sigma, k = mu */
        *sb = (float)(mu - sigma_mult * sigma);
        *se = (float)(mu + sigma_mult * sigma);
        *k = (float)mu;
    } else if (mode == LPQO_ABSMAX) {  /* Section 4.2: the absolute maximum observed */
        *sb = (float)(-amax);
        *se = (float)(amax);
        *k = 0.0f;
    } else {                           /* observed range [min, max], centred */
        *sb = (float)mn;
        *se = (float)mx;
        *k = (float)((mn + mx) / 2.0);
    }
}

static int float_cmp(const void *a, const void *b)
{
    const float x = *(const float *)a, y = *(const float *)b;
    return (x > y) - (x < y);
}

/* Outlier discard of Section 4.2 as a two-sided quantile clip: of the cnt values, sorted
 * ascending, S_b is the one of rank floor(p (cnt-1)) and S_e the one of rank
 * ceil((1-p)(cnt-1)) (ranks from 0; p = 0 gives the minimum and the maximum). */
static void quantile_range(float *vals, int64_t cnt, double p, double *lo, double *hi)
{
    qsort(vals, (size_t)cnt, sizeof(float), float_cmp);
    int64_t rl = (int64_t)floor(p * (double)(cnt - 1));
    int64_t rh = (int64_t)ceil((1.0 - p) * (double)(cnt - 1));
    if (rl < 0) rl = 0;
    if (rh > cnt - 1) rh = cnt - 1;
    *lo = (double)vals[rl];
    *hi = (double)vals[rh];
}

/* Learn (k, S_b, S_e) and m for each of d features from n vectors x[j*ld + i].
 * sigma_mult is the sigma multiplier of LPQO_GAUSS and the clipped fraction p per side
 * (0 <= p < 0.5) of LPQO_QUANTILE, whose constants are then formed as for the [min, max]
 * range.  Returns 0, or 1 if the data held a NaN/infinity or an allocation failed
 * (outputs then unspecified). */
int lpqo_calibrate(const float *x, int64_t n, int64_t ld, int d, int bits, int mode, int scope,
                   double sigma_mult, float *k, float *sb, float *se, float *m)
{
    if (scope == LPQO_PER_FEATURE || scope == LPQO_SHARED_WIDTH) {
        for (int i = 0; i < d; ++i) {
            stat_t s; stat_init(&s);
            for (int64_t j = 0; j < n; ++j) stat_add(&s, x[j * ld + i]);
            if (s.bad) return 1;
            double mu = s.sum / (double)n, ss = 0.0;
            for (int64_t j = 0; j < n; ++j) { double c = (double)x[j * ld + i] - mu; ss += c * c; }
            double sigma = sqrt(ss / (double)n);   /* maximum likelihood: divide by n */
            if (mode == LPQO_QUANTILE) {
                float *col = (float *)malloc((size_t)n * sizeof(float));
                if (!col) return 1;
                for (int64_t j = 0; j < n; ++j) col[j] = x[j * ld + i];
                quantile_range(col, n, sigma_mult, &s.mn, &s.mx);
                free(col);
            }
            constants_from(mode, sigma_mult, s.mn, s.mx, s.amax, mu, sigma, &k[i], &sb[i], &se[i]);
        }
    } else {                                       /* Section 4.1: one mu, sigma for all dimensions */
        stat_t s; stat_init(&s);
        for (int64_t j = 0; j < n; ++j)
            for (int i = 0; i < d; ++i) stat_add(&s, x[j * ld + i]);
        if (s.bad) return 1;
        double cnt = (double)n * (double)d, mu = s.sum / cnt, ss = 0.0;
        for (int64_t j = 0; j < n; ++j)
            for (int i = 0; i < d; ++i) { double c = (double)x[j * ld + i] - mu; ss += c * c; }
        double sigma = sqrt(ss / cnt);
        if (mode == LPQO_QUANTILE) {
            float *all = (float *)malloc((size_t)n * (size_t)d * sizeof(float));
            if (!all) return 1;
            for (int64_t j = 0; j < n; ++j)
                for (int i = 0; i < d; ++i) all[j * d + i] = x[j * ld + i];
            quantile_range(all, n * (int64_t)d, sigma_mult, &s.mn, &s.mx);
            free(all);
        }
        float k0, sb0, se0;
        constants_from(mode, sigma_mult, s.mn, s.mx, s.amax, mu, sigma, &k0, &sb0, &se0);
        for (int i = 0; i < d; ++i) { k[i] = k0; sb[i] = sb0; se[i] = se0; }
    }
    if (scope == LPQO_SHARED_WIDTH) {
        /* Offsets stay per dimension, the scale becomes common: every range keeps its centre
         * and takes the half-width of the widest one, so that one code step is the same length
         * in every dimension and the squared distance of codes weighs all of them alike. */
        double half = 0.0;
        for (int i = 0; i < d; ++i) {
            double h = ((double)se[i] - (double)sb[i]) / 2.0;
            if (h > half) half = h;
        }
        for (int i = 0; i < d; ++i) {
            double centre = ((double)sb[i] + (double)se[i]) / 2.0;
            sb[i] = (float)(centre - half);
            se[i] = (float)(centre + half);
        }
    }
    lpqo_derive_m(sb, se, d, bits, m);
    return 0;
}

/* Equation 1 for one value; the un-stored integer (may be +2^(B-1)). */
static int quantize_one(float x, float k, float sb, float se, float m, int bits)
{
    const int half = 1 << (bits - 1);
    if (!(se > sb)) return 0;           /* empty range: nothing to resolve */
    if (isnan(x)) return 0;
    if (x < sb) return -half;
    if (x > se) return half;
    volatile float diff = x - k;        /* volatile: two separately rounded fp32 operations */
    volatile float t = diff * m;
    float f = floorf(t);
    int r = (f >= (float)half) ? half : (f <= (float)(-half)) ? -half : (int)f;
    return r;
}

/* Codes for n vectors; one byte per code; norms[j] = sum_i code^2 if norms != NULL. */
void lpqo_encode(const float *x, int64_t n, int64_t ld, int d, int bits, const float *k,
                 const float *sb, const float *se, const float *m, int8_t *codes, int64_t ldc,
                 int32_t *norms)
{
    for (int64_t j = 0; j < n; ++j) {
        int64_t nn = 0;
        for (int i = 0; i < d; ++i) {
            int r = quantize_one(x[j * ld + i], k[i], sb[i], se[i], m[i], bits);
            if (r > 127) r = 127;       /* a byte cannot hold +128 */
            codes[j * ldc + i] = (int8_t)r;
            nn += (int64_t)r * r;
        }
        if (norms) norms[j] = (int32_t)nn;
    }
}

int32_t lpqo_dist_l2sq(const int8_t *a, const int8_t *b, int d)
{
    int64_t s = 0;
    for (int i = 0; i < d; ++i) { int64_t t = (int64_t)a[i] - (int64_t)b[i]; s += t * t; }
    return (int32_t)s;
}

int32_t lpqo_dist_ip(const int8_t *a, const int8_t *b, int d)
{
    int64_t s = 0;
    for (int i = 0; i < d; ++i) s += (int64_t)a[i] * (int64_t)b[i];
    return (int32_t)s;
}

typedef struct { int64_t key; int32_t id; } ipair_t;   /* smaller key = nearer */

static int ipair_cmp(const void *pa, const void *pb)
{
    const ipair_t *a = (const ipair_t *)pa, *b = (const ipair_t *)pb;
    if (a->key != b->key) return a->key < b->key ? -1 : 1;
    return (a->id > b->id) - (a->id < b->id);
}

/* For each query: all n distances, a full sort by (nearness, id), the first k.
 * L2SQ: ascending distance is reported; IP: descending inner product is reported.
 * Returns 0, or 1 on allocation failure. */
int lpqo_search_i8(const int8_t *codes, int64_t n, int64_t ldc, const int8_t *q, int64_t nq,
                   int64_t ldq, int d, int k, int metric, int32_t *ids, int32_t *dists,
                   int threads)
{
    int fail = 0;
    (void)threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads > 0 ? threads : 1)
#endif
    for (int64_t i = 0; i < nq; ++i) {
        ipair_t *p = (ipair_t *)malloc((size_t)n * sizeof(ipair_t));
        if (!p) { fail = 1; continue; }
        for (int64_t j = 0; j < n; ++j) {
            int32_t v = (metric == LPQO_L2SQ) ? lpqo_dist_l2sq(q + i * ldq, codes + j * ldc, d)
                                              : lpqo_dist_ip(q + i * ldq, codes + j * ldc, d);
            p[j].key = (metric == LPQO_L2SQ) ? (int64_t)v : -(int64_t)v;
            p[j].id = (int32_t)j;
        }
        qsort(p, (size_t)n, sizeof(ipair_t), ipair_cmp);
        for (int r = 0; r < k; ++r) {
            ids[i * k + r] = p[r].id;
            dists[i * k + r] = (int32_t)((metric == LPQO_L2SQ) ? p[r].key : -p[r].key);
        }
        free(p);
    }
    return fail;
}

typedef struct { double key; int32_t id; } dpair_t;

static int dpair_cmp(const void *pa, const void *pb)
{
    const dpair_t *a = (const dpair_t *)pa, *b = (const dpair_t *)pb;
    if (a->key != b->key) return a->key < b->key ? -1 : 1;
    return (a->id > b->id) - (a->id < b->id);
}

/* Exact search on the original vectors (the set S_E of Section 5.3): binary64
 * sums, ranked on the binary64 value, reported rounded to binary32. */
int lpqo_search_f32(const float *x, int64_t n, int64_t ldx, const float *q, int64_t nq,
                    int64_t ldq, int d, int k, int metric, int32_t *ids, float *dists,
                    int threads)
{
    int fail = 0;
    (void)threads;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads > 0 ? threads : 1)
#endif
    for (int64_t i = 0; i < nq; ++i) {
        dpair_t *p = (dpair_t *)malloc((size_t)n * sizeof(dpair_t));
        if (!p) { fail = 1; continue; }
        for (int64_t j = 0; j < n; ++j) {
            double s = 0.0;
            for (int t = 0; t < d; ++t) {
                double a = (double)q[i * ldq + t], b = (double)x[j * ldx + t];
                if (metric == LPQO_L2SQ) s += (a - b) * (a - b); else s += a * b;
            }
            p[j].key = (metric == LPQO_L2SQ) ? s : -s;
            p[j].id = (int32_t)j;
        }
        qsort(p, (size_t)n, sizeof(dpair_t), dpair_cmp);
        for (int r = 0; r < k; ++r) {
            ids[i * k + r] = p[r].id;
            dists[i * k + r] = (float)((metric == LPQO_L2SQ) ? p[r].key : -p[r].key);
        }
        free(p);
    }
    return fail;
}

/* Integer distances between each query and the items its list names (the distance
 * routine that Section 5.2 swaps into graph indexes: phi(Q(q), Q(x_id)) for given ids).
 * out[i][j] = phi(query i, item ids[i][j]); a negative id gives INT32_MAX (L2SQ) or
 * INT32_MIN (IP), i.e. "infinitely far". */
void lpqo_gather_dist(const int8_t *codes, int64_t ldc, const int8_t *q, int64_t nq, int64_t ldq,
                      int d, const int32_t *ids, int m, int metric, int32_t *out)
{
    for (int64_t i = 0; i < nq; ++i)
        for (int j = 0; j < m; ++j) {
            int32_t id = ids[i * m + j];
            if (id < 0) out[i * m + j] = (metric == LPQO_L2SQ) ? INT32_MAX : INT32_MIN;
            else out[i * m + j] = (metric == LPQO_L2SQ) ? lpqo_dist_l2sq(q + i * ldq, codes + (int64_t)id * ldc, d)
                                                        : lpqo_dist_ip(q + i * ldq, codes + (int64_t)id * ldc, d);
        }
}

/* Re-rank of a candidate list on the original vectors (second stage that recovers the
 * recall lost to quantization, Section 5.3's 2-6 % loss): for each query the exact
 * distance (binary64 sums) to each of its kc candidates, sorted by (nearness, id),
 * the first k reported (distance rounded to binary32).  Negative ids are skipped;
 * missing results are id -1 with distance +inf (L2SQ) / -inf (IP). */
int lpqo_rerank_f32(const float *x, int64_t ldx, const float *q, int64_t nq, int64_t ldq, int d,
                    const int32_t *cand, int kc, int k, int metric, int32_t *ids, float *dists)
{
    dpair_t *p = (dpair_t *)malloc((size_t)(kc > 0 ? kc : 1) * sizeof(dpair_t));
    if (!p) return 1;
    for (int64_t i = 0; i < nq; ++i) {
        int cnt = 0;
        for (int j = 0; j < kc; ++j) {
            int32_t id = cand[i * kc + j];
            if (id < 0) continue;
            double s = 0.0;
            for (int t = 0; t < d; ++t) {
                double a = (double)q[i * ldq + t], b = (double)x[(int64_t)id * ldx + t];
                if (metric == LPQO_L2SQ) s += (a - b) * (a - b); else s += a * b;
            }
            p[cnt].key = (metric == LPQO_L2SQ) ? s : -s;
            p[cnt].id = id;
            ++cnt;
        }
        qsort(p, (size_t)cnt, sizeof(dpair_t), dpair_cmp);
        for (int r = 0; r < k; ++r) {
            if (r < cnt) {
                ids[i * k + r] = p[r].id;
                dists[i * k + r] = (float)((metric == LPQO_L2SQ) ? p[r].key : -p[r].key);
            } else {
                ids[i * k + r] = -1;
                dists[i * k + r] = (metric == LPQO_L2SQ) ? INFINITY : -INFINITY;
            }
        }
    }
    free(p);
    return 0;
}

/* Mean over queries of |approx intersect exact| / k (Section 5.3). */
double lpqo_recall(const int32_t *approx, const int32_t *exact, int64_t nq, int k)
{
    double acc = 0.0;
    for (int64_t i = 0; i < nq; ++i) {
        int hit = 0;
        for (int a = 0; a < k; ++a)
            for (int e = 0; e < k; ++e)
                if (approx[i * k + a] == exact[i * k + e]) { ++hit; break; }
        acc += (double)hit / (double)k;
    }
    return nq > 0 ? acc / (double)nq : 0.0;
}

int lpqo_max_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}
