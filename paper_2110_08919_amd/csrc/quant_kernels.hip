// Quantizer kernels: per-feature range statistics (calibration) and the clamped linear
// encode of Equation 1, with the integer norms of the codes.  All of them stream the fp32
// matrix once with coalesced reads and are bound by HBM bandwidth.
#include "lpq_internal.h"

namespace lpq {

namespace {

constexpr int CAL_THREADS = 256;
constexpr int CAL_WAVES = CAL_THREADS / 64;
constexpr int CAL_EXTRA_ROWS = 16;   // partial rows beyond the per-block ones: the first level of the column reduction

int calib_blocks(int d)
{
    int64_t g = (int64_t(1) << 20) / d;
    if (g > 1024) g = 1024;
    if (g < 16) g = 16;
    return (int)g;
}

// Scratch: per-block partial results and the reduced per-column statistics.
struct CalibScratch {
    float *pmn, *pmx;   // [G + CAL_EXTRA_ROWS][d]
    double *psum;       // [G + CAL_EXTRA_ROWS][d]  (pass 1: sum x; pass 2: sum (x - mu)^2)
    double *csum, *css; // [d] column totals of the two passes
    double *mu;         // [d]
    float *mn, *mx;     // [d]
    // quantile selection: per column (one column when pooled) and per target (low, high rank)
    unsigned long long *qhist;   // [d][2][256] counts of the current byte among the still matching values
    unsigned long long *qrank;   // [2][d] rank still to go inside the matching values
    uint32_t *qprefix;           // [2][d] the bytes of the answer decided so far (sortable image)
};

CalibScratch carve(void *scratch, int d)
{
    const int64_t G = calib_blocks(d);
    char *p = (char *)scratch;
    CalibScratch s;
    s.psum = (double *)p; p += sizeof(double) * (G + CAL_EXTRA_ROWS) * d;
    s.csum = (double *)p; p += sizeof(double) * d;
    s.css = (double *)p;  p += sizeof(double) * d;
    s.mu = (double *)p;   p += sizeof(double) * d;
    s.pmn = (float *)p;   p += sizeof(float) * (G + CAL_EXTRA_ROWS) * d;
    s.pmx = (float *)p;   p += sizeof(float) * (G + CAL_EXTRA_ROWS) * d;
    s.mn = (float *)p;    p += sizeof(float) * d;
    s.mx = (float *)p;    p += sizeof(float) * d;
    p = (char *)(((uintptr_t)p + 15) & ~uintptr_t(15));
    s.qhist = (unsigned long long *)p;  p += sizeof(unsigned long long) * 512 * (size_t)d;
    s.qrank = (unsigned long long *)p;  p += sizeof(unsigned long long) * 2 * (size_t)d;
    s.qprefix = (uint32_t *)p;
    return s;
}

// One block reduces rows [b*R, (b+1)*R); a wave reads 64 consecutive columns of one row
// per load (256 contiguous bytes), four rows in flight.
template <int PASS>
__global__ __launch_bounds__(CAL_THREADS) void calib_reduce_kernel(
    const float *__restrict__ x, int64_t n, int64_t ld, int d, int64_t rows_per_block,
    const double *__restrict__ mu, float *__restrict__ pmn, float *__restrict__ pmx,
    double *__restrict__ psum, int *__restrict__ nonfinite)
{
    __shared__ float s_mn[CAL_WAVES][64], s_mx[CAL_WAVES][64];
    __shared__ double s_sum[CAL_WAVES][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r1 = (r0 + rows_per_block < n) ? r0 + rows_per_block : n;
    for (int c0 = 0; c0 < d; c0 += 64) {
        const int c = c0 + lane;
        const bool live = c < d;
        float mn = INFINITY, mx = -INFINITY;
        double sum = 0.0;
        bool bad = false;
        const double m = (PASS == 2 && live) ? mu[c] : 0.0;
        for (int64_t r = r0 + wave; r < r1; r += 4 * CAL_WAVES) {
            float v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t rr = r + (int64_t)u * CAL_WAVES;
                v[u] = (live && rr < r1) ? x[rr * ld + c] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t rr = r + (int64_t)u * CAL_WAVES;
                if (live && rr < r1) {
                    if (PASS == 1) {
                        if (!isfinite(v[u])) {
                            bad = true;
                        } else {
                            mn = fminf(mn, v[u]);
                            mx = fmaxf(mx, v[u]);
                            sum += (double)v[u];
                        }
                    } else {
                        const double t = (double)v[u] - m;
                        sum += t * t;
                    }
                }
            }
        }
        if (PASS == 1 && bad) atomicOr(nonfinite, 1);
        s_mn[wave][lane] = mn;
        s_mx[wave][lane] = mx;
        s_sum[wave][lane] = sum;
        __syncthreads();
        if (wave == 0 && live) {
            for (int w = 1; w < CAL_WAVES; ++w) {
                mn = fminf(mn, s_mn[w][lane]);
                mx = fmaxf(mx, s_mx[w][lane]);
                sum += s_sum[w][lane];
            }
            const int64_t o = (int64_t)blockIdx.x * d + c;
            if (PASS == 1) { pmn[o] = mn; pmx[o] = mx; }
            psum[o] = sum;
        }
        __syncthreads();
    }
}

// The same reduction with 16-byte loads, for rows that allow them (d and the row stride multiples
// of 4 floats, 16-byte aligned base): LPR lanes share a row, each owning 4 consecutive columns, so a
// wave reads 64 / LPR rows per load and four such loads are in flight per lane (64 bytes).
template <int PASS>
__global__ __launch_bounds__(CAL_THREADS) void calib_reduce_vec_kernel(
    const float *__restrict__ x, int64_t n, int64_t ld, int d, int lpr, int64_t rows_per_block,
    const double *__restrict__ mu, float *__restrict__ pmn, float *__restrict__ pmx,
    double *__restrict__ psum, int *__restrict__ nonfinite)
{
    __shared__ float s_mn[CAL_WAVES][64][4], s_mx[CAL_WAVES][64][4];
    __shared__ double s_sum[CAL_WAVES][64][4];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int cg = lane % lpr, rsel = lane / lpr, rpw = 64 / lpr;   // column group, row slot, rows per wave and load
    const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
    const int64_t r1 = (r0 + rows_per_block < n) ? r0 + rows_per_block : n;
    const int64_t rstep = (int64_t)CAL_WAVES * rpw;
    for (int c0 = 0; c0 < d; c0 += 4 * lpr) {
        const int c = c0 + 4 * cg;
        const bool live = c < d;   // d is a multiple of 4: a live lane owns 4 real columns
        float mn[4], mx[4];
        double sum[4], m[4];
        bool bad = false;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            mn[e] = INFINITY; mx[e] = -INFINITY; sum[e] = 0.0;
            m[e] = (PASS == 2 && live) ? mu[c + e] : 0.0;
        }
        for (int64_t r = r0 + (int64_t)wave * rpw + rsel; r < r1; r += 4 * rstep) {
            float4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t rr = r + u * rstep;
                v[u] = (live && rr < r1) ? *reinterpret_cast<const float4 *>(x + rr * ld + c) : float4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int64_t rr = r + u * rstep;
                if (live && rr < r1) {
                    const float a[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        if (PASS == 1) {
                            if (!isfinite(a[e])) {
                                bad = true;
                            } else {
                                mn[e] = fminf(mn[e], a[e]);
                                mx[e] = fmaxf(mx[e], a[e]);
                                sum[e] += (double)a[e];
                            }
                        } else {
                            const double t = (double)a[e] - m[e];
                            sum[e] += t * t;
                        }
                    }
                }
            }
        }
        if (PASS == 1 && bad) atomicOr(nonfinite, 1);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            s_mn[wave][lane][e] = mn[e];
            s_mx[wave][lane][e] = mx[e];
            s_sum[wave][lane][e] = sum[e];
        }
        __syncthreads();
        if (wave == 0 && rsel == 0 && live) {   // fixed order: waves, then row slots
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                float a = INFINITY, b = -INFINITY;
                double t = 0.0;
                for (int w = 0; w < CAL_WAVES; ++w)
                    for (int rs = 0; rs < rpw; ++rs) {
                        a = fminf(a, s_mn[w][rs * lpr + cg][e]);
                        b = fmaxf(b, s_mx[w][rs * lpr + cg][e]);
                        t += s_sum[w][rs * lpr + cg][e];
                    }
                const int64_t o = (int64_t)blockIdx.x * d + c + e;
                if (PASS == 1) { pmn[o] = a; pmx[o] = b; }
                psum[o] = t;
            }
        }
        __syncthreads();
    }
}

__device__ inline double block_sum(double v, double *sh)
{
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int s = CAL_THREADS / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] += sh[threadIdx.x + s];
        __syncthreads();
    }
    const double r = sh[0];
    __syncthreads();
    return r;
}
__device__ inline double block_max(double v, double *sh)
{
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int s = CAL_THREADS / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] = fmax(sh[threadIdx.x], sh[threadIdx.x + s]);
        __syncthreads();
    }
    const double r = sh[0];
    __syncthreads();
    return r;
}
__device__ inline float block_min(float v, float *sh)
{
    sh[threadIdx.x] = v;
    __syncthreads();
    for (int s = CAL_THREADS / 2; s > 0; s >>= 1) {
        if ((int)threadIdx.x < s) sh[threadIdx.x] = fminf(sh[threadIdx.x], sh[threadIdx.x + s]);
        __syncthreads();
    }
    const float r = sh[0];
    __syncthreads();
    return r;
}

// Column totals of partial rows [g_begin, g_begin + count): workgroup (x, y) takes 64 columns and
// the y-th of gridDim.y equal slices of the rows; its 16 waves share the slice and combine through
// LDS; the result goes to row y of the outputs.  Two levels (COL_PARTS slices, then their COL_PARTS
// results) keep the summation order fixed while spreading the G x d partials over 16 times as many
// workgroups.  pmn / pmx may be null (second pass: sums only).
constexpr int COL_WAVES = 16;
constexpr int COL_PARTS = 16;
__global__ __launch_bounds__(COL_WAVES * 64) void calib_colreduce_kernel(
    int g_begin, int count, int d, const float *__restrict__ pmn, const float *__restrict__ pmx,
    const double *__restrict__ psum, float *__restrict__ mn_out, float *__restrict__ mx_out, double *__restrict__ sum_out)
{
    __shared__ float s_mn[COL_WAVES][64], s_mx[COL_WAVES][64];
    __shared__ double s_sum[COL_WAVES][64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int c = blockIdx.x * 64 + lane;
    const int per = (count + (int)gridDim.y - 1) / (int)gridDim.y;
    const int g0 = g_begin + (int)blockIdx.y * per;
    const int g1 = (g0 + per < g_begin + count) ? g0 + per : g_begin + count;
    float mn = INFINITY, mx = -INFINITY;
    double sum = 0.0;
    if (c < d) {
        for (int g = g0 + wave; g < g1; g += COL_WAVES) {
            const int64_t o = (int64_t)g * d + c;
            if (pmn) { mn = fminf(mn, pmn[o]); mx = fmaxf(mx, pmx[o]); }
            sum += psum[o];
        }
    }
    s_mn[wave][lane] = mn;
    s_mx[wave][lane] = mx;
    s_sum[wave][lane] = sum;
    __syncthreads();
    if (wave == 0 && c < d) {
        for (int w = 1; w < COL_WAVES; ++w) {
            mn = fminf(mn, s_mn[w][lane]);
            mx = fmaxf(mx, s_mx[w][lane]);
            sum += s_sum[w][lane];
        }
        const int64_t o = (int64_t)blockIdx.y * d + c;
        if (mn_out) { mn_out[o] = mn; mx_out[o] = mx; }
        sum_out[o] = sum;
    }
}

// Pass-1 finalisation from the column totals; GLOBAL scope pools all columns.  In place on mn / mx.
__global__ __launch_bounds__(CAL_THREADS) void calib_stats_kernel(
    int d, int64_t n, int scope, float *__restrict__ mn_io, float *__restrict__ mx_io,
    const double *__restrict__ csum, double *__restrict__ mu_out)
{
    __shared__ double shd[CAL_THREADS];
    __shared__ float shf[CAL_THREADS];
    if (scope != LPQ_SCOPE_GLOBAL) {
        for (int c = threadIdx.x; c < d; c += CAL_THREADS) mu_out[c] = csum[c] / (double)n;
        return;
    }
    float gmn = INFINITY, gmx = -INFINITY;
    double gsum = 0.0;
    for (int c = threadIdx.x; c < d; c += CAL_THREADS) {
        gmn = fminf(gmn, mn_io[c]);
        gmx = fmaxf(gmx, mx_io[c]);
        gsum += csum[c];
    }
    gmn = block_min(gmn, shf);
    gmx = -block_min(-gmx, shf);
    gsum = block_sum(gsum, shd);
    const double mu = gsum / ((double)n * (double)d);
    for (int c = threadIdx.x; c < d; c += CAL_THREADS) {
        mn_io[c] = gmn;
        mx_io[c] = gmx;
        mu_out[c] = mu;
    }
}

// ------------------------------------------------------------- quantile selection --
// Exact order statistics by radix selection on an order-preserving 32-bit image of the floats:
// four passes from the most significant byte; each pass counts, per column and per target
// rank, the values that still match the bytes decided so far, then the bin holding the rank
// fixes the next byte.
__device__ __forceinline__ uint32_t float_sortable_u32(float f)
{
    const uint32_t u = (uint32_t)__float_as_int(f);
    return (u >> 31) ? ~u : (u | 0x80000000u);
}
__device__ __forceinline__ float sortable_u32_float(uint32_t u)
{
    return __int_as_float((int)((u >> 31) ? (u & 0x7fffffffu) : ~u));
}

__global__ void quantile_init_kernel(int cols, unsigned long long rank_lo, unsigned long long rank_hi,
                                     unsigned long long *qrank, uint32_t *qprefix, unsigned long long *qhist)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < cols) {
        qrank[i] = rank_lo; qrank[cols + i] = rank_hi;
        qprefix[i] = 0u; qprefix[cols + i] = 0u;
    }
    for (int j = i; j < cols * 512; j += gridDim.x * blockDim.x) qhist[j] = 0ull;
}

// One pass of the radix selection over a tile of COLS columns x rows_per_block rows.  A lane owns
// ONE column (lane % COLS) and every (256 / COLS)-th row of the tile, so the lanes of a load read
// COLS consecutive floats of a row (256 or 128 contiguous bytes) and no two lanes of a wave's
// first COLS lanes ever count into the same histogram; the histograms of a column are 257 words
// apart, so equal bins of neighbouring columns - the common case, the exponent byte of most values
// is the same - fall into different LDS banks.  NT = 1 is the first pass: no byte is decided yet,
// both target ranks see the same counts, one histogram per column serves both.  NT = 2: a value
// counts for a target if it matches the bytes decided for that target so far.  Eight loads of a
// lane are in flight before their counts are taken.
// pooled: all d columns count into column 0 (one set of constants for all dimensions).
constexpr int QH_STRIDE = 257;
template <int COLS, int NT>
__global__ __launch_bounds__(256) void quantile_hist_kernel(
    const float *__restrict__ x, int64_t n, int64_t ld, int d, int64_t rows_per_block, int shift,
    int pooled, int cols, const uint32_t *__restrict__ qprefix, unsigned long long *__restrict__ qhist)
{
    extern __shared__ uint32_t qh_lds[];   // [COLS][NT][QH_STRIDE]
    constexpr int RL = 256 / COLS, U = 8;
    for (int i = threadIdx.x; i < COLS * NT * QH_STRIDE; i += 256) qh_lds[i] = 0u;
    __syncthreads();
    const int cl = threadIdx.x % COLS, rl = threadIdx.x / COLS;
    const int c = blockIdx.y * COLS + cl;
    const int cg = pooled ? 0 : c;
    uint32_t *h0 = qh_lds + (size_t)cl * NT * QH_STRIDE, *h1 = h0 + (NT - 1) * QH_STRIDE;
    if (c < d) {
        const uint32_t keep = NT == 1 ? 0u : (0xFFFFFFFFu << (shift + 8));   // the bytes already decided
        const uint32_t p0 = NT == 1 ? 0u : qprefix[cg], p1 = NT == 1 ? 0u : qprefix[cols + cg];
        const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
        const int64_t r1 = (r0 + rows_per_block < n) ? r0 + rows_per_block : n;
        const float *col = x + c;
        for (int64_t r = r0 + rl; r < r1; r += (int64_t)RL * U) {
            uint32_t key[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t rr = r + (int64_t)u * RL;
                key[u] = float_sortable_u32(col[(rr < r1 ? rr : r) * ld]);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (r + (int64_t)u * RL >= r1) break;
                const int b = (int)((key[u] >> shift) & 255u);
                if (NT == 1) {
                    atomicAdd(&h0[b], 1u);
                } else {
                    if (((key[u] ^ p0) & keep) == 0u) atomicAdd(&h0[b], 1u);
                    if (((key[u] ^ p1) & keep) == 0u) atomicAdd(&h1[b], 1u);
                }
            }
        }
    }
    __syncthreads();
    for (int i = threadIdx.x; i < COLS * NT * 256; i += 256) {
        const int lc = i / (NT * 256), t = (i / 256) % NT, b = i % 256;
        const uint32_t v = qh_lds[(size_t)(lc * NT + t) * QH_STRIDE + b];
        const int gc = blockIdx.y * COLS + lc;
        if (v && gc < d) {
            unsigned long long *hh = qhist + (size_t)(pooled ? 0 : gc) * 512;
            if (NT == 1) {   // the same counts for both targets
                atomicAdd(&hh[b], (unsigned long long)v);
                atomicAdd(&hh[256 + b], (unsigned long long)v);
            } else {
                atomicAdd(&hh[t * 256 + b], (unsigned long long)v);
            }
        }
    }
}

// The same pass for rows that allow 16-byte loads (d and ld multiples of 4, 16-byte aligned base):
// 1024 threads, one workgroup per CU with all the histograms of a COLS-column tile (COLS x NT x 257
// words, 132 KB); a lane owns FOUR consecutive columns (one float4 per row) and every
// (1024 / (COLS / 4))-th row, four loads in flight: 64 bytes per lane, 64 KB per CU, which is what
// it takes to keep HBM busy (with one float per lane and 512 threads per CU the pass ran at 1.7 TB/s).
// Column c of the tile counts into histogram slot (c % 4) * (COLS / 4) + c / 4, so that the lanes of a
// row, which handle columns 4j + i in their i-th update, hit consecutive slots and hence different
// banks when their bins are equal.  pooled: the tile's histograms are summed in LDS before the flush,
// so a workgroup sends 256 NT global atomics instead of 256 NT COLS to the one global histogram.
template <int COLS, int NT>
__global__ __launch_bounds__(1024) void quantile_hist_vec_kernel(
    const float *__restrict__ x, int64_t n, int64_t ld, int d, int64_t rows_per_block, int shift,
    int pooled, int cols, const uint32_t *__restrict__ qprefix, unsigned long long *__restrict__ qhist)
{
    extern __shared__ uint32_t qh_lds[];   // [COLS slots][NT][QH_STRIDE]
    constexpr int LPR = COLS / 4, RL = 1024 / LPR, U = 4;
    for (int i = threadIdx.x; i < COLS * NT * QH_STRIDE; i += 1024) qh_lds[i] = 0u;
    __syncthreads();
    const int jl = threadIdx.x % LPR, rl = threadIdx.x / LPR;
    const int c0 = blockIdx.y * COLS + 4 * jl;          // first of this lane's four columns
    if (c0 < d) {                                       // d % 4 == 0: all four exist
        const uint32_t keep = NT == 1 ? 0u : (0xFFFFFFFFu << (shift + 8));   // the bytes already decided
        uint32_t p0[4], p1[4];
        uint32_t *h[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int cg = pooled ? 0 : c0 + i;
            p0[i] = NT == 1 ? 0u : qprefix[cg];
            p1[i] = NT == 1 ? 0u : qprefix[cols + cg];
            h[i] = qh_lds + (size_t)(i * LPR + jl) * NT * QH_STRIDE;
        }
        const int64_t r0 = (int64_t)blockIdx.x * rows_per_block;
        const int64_t r1 = (r0 + rows_per_block < n) ? r0 + rows_per_block : n;
        const float *base = x + c0;
        for (int64_t r = r0 + rl; r < r1; r += (int64_t)RL * U) {
            float4 v[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int64_t rr = r + (int64_t)u * RL;
                v[u] = *reinterpret_cast<const float4 *>(base + (rr < r1 ? rr : r) * ld);
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (r + (int64_t)u * RL >= r1) break;
                const float f[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const uint32_t key = float_sortable_u32(f[i]);
                    const int b = (int)((key >> shift) & 255u);
                    if (NT == 1) {
                        atomicAdd(&h[i][b], 1u);
                    } else {
                        if (((key ^ p0[i]) & keep) == 0u) atomicAdd(&h[i][b], 1u);
                        if (((key ^ p1[i]) & keep) == 0u) atomicAdd(&h[i][QH_STRIDE + b], 1u);
                    }
                }
            }
        }
    }
    __syncthreads();
    if (pooled) {   // one histogram for the whole tile: bins summed over the slots first
        for (int i = threadIdx.x; i < NT * 256; i += 1024) {
            const int t = i / 256, b = i % 256;
            unsigned long long sum = 0ull;
            for (int sl = 0; sl < COLS; ++sl) sum += qh_lds[(size_t)(sl * NT + t) * QH_STRIDE + b];
            if (sum) {
                if (NT == 1) { atomicAdd(&qhist[b], sum); atomicAdd(&qhist[256 + b], sum); }
                else atomicAdd(&qhist[t * 256 + b], sum);
            }
        }
        return;
    }
    for (int i = threadIdx.x; i < COLS * NT * 256; i += 1024) {
        const int sl = i / (NT * 256), t = (i / 256) % NT, b = i % 256;
        const uint32_t v = qh_lds[(size_t)(sl * NT + t) * QH_STRIDE + b];
        const int gc = blockIdx.y * COLS + 4 * (sl % LPR) + sl / LPR;   // the column behind slot sl
        if (v && gc < d) {
            unsigned long long *hh = qhist + (size_t)gc * 512;
            if (NT == 1) {   // the same counts for both targets
                atomicAdd(&hh[b], (unsigned long long)v);
                atomicAdd(&hh[256 + b], (unsigned long long)v);
            } else {
                atomicAdd(&hh[t * 256 + b], (unsigned long long)v);
            }
        }
    }
}

// One wave per (column, target): the bin that holds the rank decides the next byte.  Lane l sums bins
// 4l .. 4l + 3, an inclusive scan over the lanes finds the lane whose bins hold the rank, that lane
// finds the bin.  (One thread walking the 256 bins took 24 us per pass.)
__global__ __launch_bounds__(256) void quantile_pick_kernel(int cols, int shift, unsigned long long *qrank, uint32_t *qprefix,
                                                            unsigned long long *qhist)
{
    const int lane = threadIdx.x & 63;
    const int i = blockIdx.x * 4 + (threadIdx.x >> 6);   // wave-uniform
    if (i >= cols * 2) return;
    const int c = i >> 1, t = i & 1;
    unsigned long long *hh = qhist + ((size_t)c * 2 + t) * 256;
    const unsigned long long rank = qrank[t * cols + c];
    unsigned long long v[4], mine = 0ull;
#pragma unroll
    for (int j = 0; j < 4; ++j) { v[j] = hh[4 * lane + j]; mine += v[j]; }
    unsigned long long incl = mine;                      // sum over lanes 0 .. lane
#pragma unroll
    for (int o = 1; o < 64; o <<= 1) {
        const unsigned long long up = __shfl_up(incl, o, 64);
        if (lane >= o) incl += up;
    }
    // the first lane whose inclusive sum exceeds the rank holds it; if none does (cannot happen for a
    // rank below the count) the last bin is taken, as the serial walk did
    const unsigned long long has = __ballot(rank < incl);
    const int win = has ? __ffsll((unsigned long long)has) - 1 : 63;
    if (lane == win) {
        unsigned long long before = incl - mine;
        int bin = 4 * lane + 3;
        if (has) {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                if (rank < before + v[j]) { bin = 4 * lane + j; break; }
                before += v[j];
            }
        } else {
            before = incl;
        }
        qrank[t * cols + c] = rank - before;
        qprefix[t * cols + c] |= (uint32_t)bin << shift;
    }
#pragma unroll
    for (int j = 0; j < 4; ++j) hh[4 * lane + j] = 0ull;
}

__global__ void quantile_finish_kernel(int d, int pooled, int cols, const uint32_t *qprefix, float *mn, float *mx)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < d) {
        const int cg = pooled ? 0 : c;
        mn[c] = sortable_u32_float(qprefix[cg]);
        mx[c] = sortable_u32_float(qprefix[cols + cg]);
    }
}

__device__ inline float derive_m(float sb, float se, int bits)
{
    const double width = (double)se - (double)sb;
    return (width > 0.0) ? (float)(ldexp(1.0, bits) / width) : 0.0f;
}

// Constants of Equation 1 from the statistics (Sections 3.2, 4.1, 4.2).
__global__ __launch_bounds__(CAL_THREADS) void calib_params_kernel(
    int d, int64_t n, int bits, int mode, int scope, double sigma_mult,
    const float *__restrict__ mn, const float *__restrict__ mx, const double *__restrict__ mu,
    const double *__restrict__ css, float *__restrict__ params)
{
    __shared__ double shd[CAL_THREADS];
    double gss = 0.0;
    if (mode == LPQ_CALIB_GAUSS && scope == LPQ_SCOPE_GLOBAL) {
        for (int c = threadIdx.x; c < d; c += CAL_THREADS) gss += css[c];
        gss = block_sum(gss, shd);
    }
    for (int c = threadIdx.x; c < d; c += CAL_THREADS) {
        float k, sb, se;
        if (mode == LPQ_CALIB_GAUSS) {
            double ss = gss, cnt = (double)n * (double)d;
            if (scope != LPQ_SCOPE_GLOBAL) {
                ss = css[c];
                cnt = (double)n;
            }
            const double sigma = sqrt(ss / cnt);
            sb = (float)(mu[c] - sigma_mult * sigma);
            se = (float)(mu[c] + sigma_mult * sigma);
            k = (float)mu[c];
        } else if (mode == LPQ_CALIB_ABSMAX) {
            const double amax = fmax(fabs((double)mn[c]), fabs((double)mx[c]));
            sb = (float)(-amax);
            se = (float)amax;
            k = 0.0f;
        } else {
            sb = mn[c];
            se = mx[c];
            k = (float)(((double)mn[c] + (double)mx[c]) / 2.0);
        }
        params[c] = k;
        params[d + c] = sb;
        params[2 * d + c] = se;
        params[3 * d + c] = derive_m(sb, se, bits);
    }
    if (scope != LPQ_SCOPE_SHARED_WIDTH) return;
    // One width for all dimensions: every range keeps its centre and takes the half-width of
    // the widest one (binary64 arithmetic on the binary32 constants just written).
    __syncthreads();
    double half = 0.0;
    for (int c = threadIdx.x; c < d; c += CAL_THREADS)
        half = fmax(half, ((double)params[2 * d + c] - (double)params[d + c]) / 2.0);
    half = block_max(half, shd);
    for (int c = threadIdx.x; c < d; c += CAL_THREADS) {
        const double centre = ((double)params[d + c] + (double)params[2 * d + c]) / 2.0;
        const float sb = (float)(centre - half), se = (float)(centre + half);
        params[d + c] = sb;
        params[2 * d + c] = se;
        params[3 * d + c] = derive_m(sb, se, bits);
    }
}

__global__ void derive_m_kernel(float *params, int d, int bits)
{
    const int c = blockIdx.x * blockDim.x + threadIdx.x;
    if (c < d) params[3 * d + c] = derive_m(params[d + c], params[2 * d + c], bits);
}

// ------------------------------------------------------------------------- encode --
// Equation 1 for one value, in binary32 with separately rounded subtract and multiply.
// lo = -2^(B-1) and top = min(2^(B-1), 127) as floats; an empty range (S_e <= S_b) arrives here
// as sb = -inf, se = +inf, m = 0 (see column_constants), which yields 0 for every x.
__device__ inline int quantize_one(float x, float k, float sb, float se, float m, float lo, float top)
{
    const float t = __fmul_rn(__fsub_rn(x, k), m);
    // floor, clamp to the code range (the stored top code included), convert: the clamp keeps the
    // conversion in range; a NaN (from x, or from inf * 0) is replaced below
    float f = __builtin_amdgcn_fmed3f(floorf(t), lo, top);
    f = (x > se) ? top : f;
    f = (x < sb) ? lo : f;
    f = (t != t) ? 0.0f : f;
    return (int)f;
}

// Constants of column c as the encoder uses them.
__device__ inline void column_constants(const QuantParams &qp, int c, bool in, float &k, float &sb, float &se, float &m)
{
    k = in ? qp.k[c] : 0.f;
    sb = in ? qp.sb[c] : 0.f;
    se = in ? qp.se[c] : 0.f;
    m = in ? qp.m[c] : 0.f;
    if (!(se > sb)) {   // empty range: code 0 everywhere
        sb = -INFINITY;
        se = INFINITY;
        m = 0.f;
    }
}

constexpr int ENC_THREADS = 256;
constexpr int ENC_UNROLL = 4;

// TPR lanes share one row (4 columns each per step); a wave covers 64/TPR rows at once and
// ENC_UNROLL such row groups are in flight.  VEC: rows are 16-byte aligned in x and 4-byte
// aligned in codes, so float4 loads and packed 32-bit stores are used.
template <int TPR, bool VEC>
__global__ __launch_bounds__(ENC_THREADS) void encode_kernel(
    QuantParams qp, const float *__restrict__ x, int64_t n, int64_t ld, int8_t *__restrict__ codes,
    int64_t ldc, int zero_pad_to, int32_t *__restrict__ norms, int64_t n_out)
{
    // rows n .. n_out-1 (padding rows of a query tile) are written as zero codes
    constexpr int RPW = 64 / TPR;
    const int lane = threadIdx.x & 63;
    const int sub = lane % TPR, rsel = lane / TPR;
    const int d = qp.d, half = 1 << (qp.bits - 1);
    const float lo = (float)(-half), top = (float)(half < 127 ? half : 127);
    const int ngroups = (d + 3) >> 2;              // 4-column groups holding data
    const int pgroups = (zero_pad_to > d) ? ((zero_pad_to + 3) >> 2) : ngroups;
    const int64_t wave_id = ((int64_t)blockIdx.x * ENC_THREADS + threadIdx.x) >> 6;
    const int64_t nwaves = ((int64_t)gridDim.x * ENC_THREADS) >> 6;
    const bool single = pgroups <= TPR;            // each lane owns one column group: hoist constants

    float ck[4] = {0, 0, 0, 0}, cb[4] = {0, 0, 0, 0}, ce[4] = {0, 0, 0, 0}, cm[4] = {0, 0, 0, 0};
    if (single) {
#pragma unroll
        for (int j = 0; j < 4; ++j) column_constants(qp, 4 * sub + j, 4 * sub + j < d, ck[j], cb[j], ce[j], cm[j]);
    }
    for (int64_t base = wave_id * RPW * ENC_UNROLL; base < n_out; base += nwaves * RPW * ENC_UNROLL) {
        int acc[ENC_UNROLL];
#pragma unroll
        for (int u = 0; u < ENC_UNROLL; ++u) acc[u] = 0;
        for (int g0 = 0; g0 < pgroups; g0 += TPR) {
            const int g = g0 + sub;
            const int c0 = 4 * g;
            if (!single) {
#pragma unroll
                for (int j = 0; j < 4; ++j) column_constants(qp, c0 + j, c0 + j < d, ck[j], cb[j], ce[j], cm[j]);
            }
            float v[ENC_UNROLL][4];
#pragma unroll
            for (int u = 0; u < ENC_UNROLL; ++u) {
                const int64_t r = base + u * RPW + rsel;
                const bool rowok = r < n && g < ngroups;
                if (VEC && rowok && c0 + 3 < d) {
                    const float4 t = *reinterpret_cast<const float4 *>(x + r * ld + c0);
                    v[u][0] = t.x; v[u][1] = t.y; v[u][2] = t.z; v[u][3] = t.w;
                } else {
#pragma unroll
                    for (int j = 0; j < 4; ++j) v[u][j] = (rowok && c0 + j < d) ? x[r * ld + c0 + j] : 0.0f;
                }
            }
#pragma unroll
            for (int u = 0; u < ENC_UNROLL; ++u) {
                const int64_t r = base + u * RPW + rsel;
                if (r < n_out && g < pgroups) {
                    int q[4];
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        q[j] = (c0 + j < d && r < n) ? quantize_one(v[u][j], ck[j], cb[j], ce[j], cm[j], lo, top) : 0;
                        acc[u] += q[j] * q[j];
                    }
                    const int lim = (zero_pad_to > d) ? zero_pad_to : d;
                    if (VEC && c0 + 3 < lim) {
                        const uint32_t w = (uint32_t)(q[0] & 255) | ((uint32_t)(q[1] & 255) << 8) |
                                           ((uint32_t)(q[2] & 255) << 16) | ((uint32_t)(q[3] & 255) << 24);
                        *reinterpret_cast<uint32_t *>(codes + r * ldc + c0) = w;
                    } else {
#pragma unroll
                        for (int j = 0; j < 4; ++j)
                            if (c0 + j < lim) codes[r * ldc + c0 + j] = (int8_t)q[j];
                    }
                }
            }
        }
        if (norms) {
#pragma unroll
            for (int u = 0; u < ENC_UNROLL; ++u) {
                int s = acc[u];
#pragma unroll
                for (int o = TPR / 2; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
                const int64_t r = base + u * RPW + rsel;
                if (sub == 0 && r < n_out) norms[r] = s;
            }
        }
    }
}

// Copy int8 rows into zero-padded rows and compute their norms; 16 lanes per row.
__global__ __launch_bounds__(256) void repack_i8_kernel(
    const int8_t *__restrict__ src, int64_t n, int64_t ld, int d, int8_t *__restrict__ dst,
    int64_t ldd, int d_pad, int32_t *__restrict__ norms, int64_t n_out)
{
    const int sub = threadIdx.x & 15;
    const int64_t r = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 4;
    int s = 0;
    if (r < n_out) {
        for (int c = sub; c < d_pad; c += 16) {
            const int v = (c < d && r < n) ? (int)src[r * ld + c] : 0;
            dst[r * ldd + c] = (int8_t)v;
            s += v * v;
        }
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (r < n_out && sub == 0 && norms) norms[r] = s;
}

// Two 4-bit codes per byte (sub-byte packing for B <= 4): byte j of a row holds code 2j in its low
// nibble and code 2j+1 in its high nibble, each stored as u = code + 8.  A nibble cannot hold +8,
// so the upper clamp value of B = 4 is stored as 7 (as a byte stores +128 as 127 at B = 8); the
// norm is that of the stored codes.  Columns d .. d_pad-1 hold code 0.  16 lanes per row.
__global__ __launch_bounds__(256) void pack4_kernel(const int8_t *__restrict__ src, int64_t n, int64_t ld, int d,
                                                    uint8_t *__restrict__ dst, int d_pad, int32_t *__restrict__ norms)
{
    const int sub = threadIdx.x & 15;
    const int64_t r = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 4;
    int s = 0;
    if (r < n) {
        for (int j = sub; j < d_pad / 2; j += 16) {
            int c0 = (2 * j < d) ? (int)src[r * ld + 2 * j] : 0;
            int c1 = (2 * j + 1 < d) ? (int)src[r * ld + 2 * j + 1] : 0;
            c0 = c0 > 7 ? 7 : (c0 < -8 ? -8 : c0);
            c1 = c1 > 7 ? 7 : (c1 < -8 ? -8 : c1);
            dst[r * (d_pad / 2) + j] = (uint8_t)((c0 + 8) | ((c1 + 8) << 4));
            s += c0 * c0 + c1 * c1;
        }
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
    if (r < n && sub == 0) norms[r] = s;
}

// Query codes in the order the packed scan's operand unpacking produces (inside every group of 16
// codes: 0 2 4 6 1 3 5 7 8 10 12 14 9 11 13 15), and the per-query term that takes the + 8 offset
// of the stored corpus codes out of the result: L2SQ |cq|^2 + 16 sum(cq), IP -8 sum(cq).  Codes are
// saturated to the nibble range [-8, 7] first.
__global__ __launch_bounds__(256) void permute_queries_kernel(const int8_t *__restrict__ q, int64_t nq_pad, int d_pad,
                                                              int l2, int8_t *__restrict__ qperm, int32_t *__restrict__ qadj)
{
    const int sub = threadIdx.x & 15;
    const int64_t r = ((int64_t)blockIdx.x * 256 + threadIdx.x) >> 4;
    int sum = 0, sq = 0;
    if (r < nq_pad) {
        for (int c = sub; c < d_pad; c += 16) {
            const int i = c & 15, g = c & ~15;
            const int h = i & 7;                                  // position inside a half of 8
            const int srci = (i & 8) | (h < 4 ? 2 * h : 2 * (h - 4) + 1);
            int v = (int)q[r * d_pad + g + srci];
            v = v > 7 ? 7 : (v < -8 ? -8 : v);   // queries saturate like the stored items
            qperm[r * d_pad + c] = (int8_t)v;
            sum += v;
            sq += v * v;
        }
    }
#pragma unroll
    for (int o = 8; o > 0; o >>= 1) { sum += __shfl_xor(sum, o, 64); sq += __shfl_xor(sq, o, 64); }
    if (r < nq_pad && sub == 0) qadj[r] = l2 ? sq + 16 * sum : -8 * sum;
}

__global__ __launch_bounds__(256) void zero_words_kernel(uint32_t *p, size_t words)
{
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < words; i += (size_t)gridDim.x * 256) p[i] = 0u;
}

// One thread per 32-item word: accumulator seeds and norm parities for items
// [32w, 32w + 32); items at or beyond n_total get the padding seed.
__global__ __launch_bounds__(256) void item_aux_kernel(
    const int32_t *__restrict__ norms, int64_t w0, int64_t w1, int64_t n_total,
    int32_t *__restrict__ cinit, uint32_t *__restrict__ parity)
{
    const int64_t w = w0 + (int64_t)blockIdx.x * 256 + threadIdx.x;
    if (w >= w1) return;
    uint32_t bits = 0;
    for (int r = 0; r < 32; ++r) {
        const int64_t j = w * 32 + r;
        int32_t ci = CINIT_PAD;
        if (j < n_total) {
            const int32_t nx = norms ? norms[j] : 0;
            ci = -((nx + 1) >> 1);
            bits |= (uint32_t)(nx & 1) << r;
        }
        cinit[j] = ci;
    }
    parity[w] = bits;
}

}  // namespace

size_t calib_scratch_bytes(int d)
{
    const size_t G = calib_blocks(d) + CAL_EXTRA_ROWS;
    return G * d * (sizeof(double) + 2 * sizeof(float)) + (size_t)d * (3 * sizeof(double) + 2 * sizeof(float)) + 256 +
           (size_t)d * (512 * sizeof(unsigned long long) + 2 * sizeof(unsigned long long) + 2 * sizeof(uint32_t));
}

hipError_t launch_calibrate(const float *x, int64_t n, int64_t ld, int d, int bits, int mode, int scope,
                            double sigma_mult, void *scratch, float *params_out, int *nonfinite_flag,
                            hipStream_t st)
{
    const int G = calib_blocks(d);
    CalibScratch s = carve(scratch, d);
    const int64_t rpb = ceil_div(n, G);
    hipError_t e = hipMemsetAsync(nonfinite_flag, 0, sizeof(int), st);
    if (e != hipSuccess) return e;
    // 16-byte loads when the rows allow them; lanes per row: the power of two that covers d / 4
    const bool vec = d % 4 == 0 && ld % 4 == 0 && (uintptr_t)x % 16 == 0;
    int lpr = 1;
    while (lpr < d / 4 && lpr < 64) lpr <<= 1;
    if (vec)
        calib_reduce_vec_kernel<1><<<G, CAL_THREADS, 0, st>>>(x, n, ld, d, lpr, rpb, nullptr, s.pmn, s.pmx, s.psum,
                                                              nonfinite_flag);
    else
        calib_reduce_kernel<1><<<G, CAL_THREADS, 0, st>>>(x, n, ld, d, rpb, nullptr, s.pmn, s.pmx, s.psum,
                                                          nonfinite_flag);
    const int cblocks = (d + 63) / 64;
    static_assert(COL_PARTS <= CAL_EXTRA_ROWS, "the first level writes COL_PARTS partial rows behind the G block rows");
    const size_t lvl = (size_t)G * d;   // first-level results live in rows G .. G + COL_PARTS - 1
    calib_colreduce_kernel<<<dim3(cblocks, COL_PARTS), COL_WAVES * 64, 0, st>>>(0, G, d, s.pmn, s.pmx, s.psum, s.pmn + lvl,
                                                                               s.pmx + lvl, s.psum + lvl);
    calib_colreduce_kernel<<<dim3(cblocks, 1), COL_WAVES * 64, 0, st>>>(G, COL_PARTS, d, s.pmn, s.pmx, s.psum, s.mn, s.mx,
                                                                       s.csum);
    calib_stats_kernel<<<1, CAL_THREADS, 0, st>>>(d, n, scope, s.mn, s.mx, s.csum, s.mu);
    if (mode == LPQ_CALIB_QUANTILE) {
        // the min/max pass above has checked the data; now the two order statistics per column
        const int pooled = scope == LPQ_SCOPE_GLOBAL, cols = pooled ? 1 : d;
        const double cnt = pooled ? (double)n * (double)d : (double)n;
        double rl = floor(sigma_mult * (cnt - 1.0)), rh = ceil((1.0 - sigma_mult) * (cnt - 1.0));
        if (rl < 0.0) rl = 0.0;
        if (rh > cnt - 1.0) rh = cnt - 1.0;
        quantile_init_kernel<<<(cols * 512 + 255) / 256, 256, 0, st>>>(cols, (unsigned long long)rl, (unsigned long long)rh,
                                                                       s.qrank, s.qprefix, s.qhist);
        // First pass: one histogram per column serves both ranks, so a workgroup takes twice the columns
        // of the later passes in the same LDS.  Rows per workgroup: 256 workgroups in all, one per CU: every
        // workgroup flushes its histograms with one global atomic per non-empty bin, which is what the
        // passes over the low bytes (all bins in use) spend their time on with more of them (1M x 128 per
        // feature, whole calibration: 1.00 / 0.88 / 0.79 / 0.72 ms with 2048 / 1024 / 512 / 256).
        constexpr size_t qlds = (size_t)64 * QH_STRIDE * sizeof(uint32_t), qlds_vec = 2 * qlds;
        static bool qattr = false;
        if (!qattr) {
            const void *kerns[4] = {reinterpret_cast<const void *>(quantile_hist_kernel<64, 1>),
                                    reinterpret_cast<const void *>(quantile_hist_kernel<32, 2>),
                                    reinterpret_cast<const void *>(quantile_hist_vec_kernel<128, 1>),
                                    reinterpret_cast<const void *>(quantile_hist_vec_kernel<64, 2>)};
            for (int i = 0; i < 4; ++i) {
                e = hipFuncSetAttribute(kerns[i], hipFuncAttributeMaxDynamicSharedMemorySize, (int)(i < 2 ? qlds : qlds_vec));
                if (e != hipSuccess) return e;
            }
            qattr = true;
        }
        for (int pass = 0; pass < 4; ++pass) {
            const int shift = 24 - 8 * pass;
            const int tile = (pass == 0 ? 64 : 32) * (vec ? 2 : 1);
            const int64_t tiles = ceil_div(d, tile);
            int64_t qrpb = round_up(ceil_div(n * tiles, 256), 64);
            if (qrpb < 1024) qrpb = 1024;
            const dim3 grid((unsigned)ceil_div(n, qrpb), (unsigned)tiles);
            if (vec && pass == 0)
                quantile_hist_vec_kernel<128, 1><<<grid, 1024, qlds_vec, st>>>(x, n, ld, d, qrpb, shift, pooled, cols, s.qprefix, s.qhist);
            else if (vec)
                quantile_hist_vec_kernel<64, 2><<<grid, 1024, qlds_vec, st>>>(x, n, ld, d, qrpb, shift, pooled, cols, s.qprefix, s.qhist);
            else if (pass == 0)
                quantile_hist_kernel<64, 1><<<grid, 256, qlds, st>>>(x, n, ld, d, qrpb, shift, pooled, cols, s.qprefix, s.qhist);
            else
                quantile_hist_kernel<32, 2><<<grid, 256, qlds, st>>>(x, n, ld, d, qrpb, shift, pooled, cols, s.qprefix, s.qhist);
            quantile_pick_kernel<<<(cols * 2 + 3) / 4, 256, 0, st>>>(cols, shift, s.qrank, s.qprefix, s.qhist);
        }
        quantile_finish_kernel<<<(d + 255) / 256, 256, 0, st>>>(d, pooled, cols, s.qprefix, s.mn, s.mx);
    }
    if (mode == LPQ_CALIB_GAUSS) {
        if (vec)
            calib_reduce_vec_kernel<2><<<G, CAL_THREADS, 0, st>>>(x, n, ld, d, lpr, rpb, s.mu, nullptr, nullptr, s.psum,
                                                                  nonfinite_flag);
        else
            calib_reduce_kernel<2><<<G, CAL_THREADS, 0, st>>>(x, n, ld, d, rpb, s.mu, nullptr, nullptr, s.psum,
                                                              nonfinite_flag);
        calib_colreduce_kernel<<<dim3(cblocks, COL_PARTS), COL_WAVES * 64, 0, st>>>(0, G, d, nullptr, nullptr, s.psum, nullptr,
                                                                                   nullptr, s.psum + lvl);
        calib_colreduce_kernel<<<dim3(cblocks, 1), COL_WAVES * 64, 0, st>>>(G, COL_PARTS, d, nullptr, nullptr, s.psum, nullptr,
                                                                           nullptr, s.css);
    }
    calib_params_kernel<<<1, CAL_THREADS, 0, st>>>(d, n, bits, mode, scope, sigma_mult, s.mn, s.mx, s.mu, s.css,
                                                   params_out);
    return hipGetLastError();
}

hipError_t launch_derive_m(float *params, int d, int bits, hipStream_t st)
{
    derive_m_kernel<<<(d + 255) / 256, 256, 0, st>>>(params, d, bits);
    return hipGetLastError();
}

template <int TPR>
static void encode_dispatch(bool vec, int blocks, hipStream_t st, const QuantParams &qp, const float *x,
                            int64_t n, int64_t ld, int8_t *codes, int64_t ldc, int zero_pad_to, int32_t *norms,
                            int64_t n_out)
{
    if (vec)
        encode_kernel<TPR, true><<<blocks, ENC_THREADS, 0, st>>>(qp, x, n, ld, codes, ldc, zero_pad_to, norms, n_out);
    else
        encode_kernel<TPR, false><<<blocks, ENC_THREADS, 0, st>>>(qp, x, n, ld, codes, ldc, zero_pad_to, norms, n_out);
}

hipError_t launch_encode(const QuantParams &qp, const float *x, int64_t n, int64_t ld, int8_t *codes,
                         int64_t ldc, int zero_pad_to, int32_t *norms, hipStream_t st, int64_t n_out)
{
    if (n_out < n) n_out = n;
    if (n_out <= 0) return hipSuccess;
    const int lim = zero_pad_to > qp.d ? zero_pad_to : qp.d;
    const int groups = (lim + 3) / 4;
    int tpr = 1;
    while (tpr < groups && tpr < 64) tpr <<= 1;
    const bool vec = ((uintptr_t)x % 16 == 0) && (ld % 4 == 0) && ((uintptr_t)codes % 4 == 0) && (ldc % 4 == 0);
    const int rpw = 64 / tpr;
    int64_t waves = ceil_div(n_out, (int64_t)rpw * ENC_UNROLL);
    int64_t blocks = ceil_div(waves, ENC_THREADS / 64);
    if (blocks > 256 * 16) blocks = 256 * 16;
    switch (tpr) {
    case 1: encode_dispatch<1>(vec, (int)blocks, st, qp, x, n, ld, codes, ldc, zero_pad_to, norms, n_out); break;
    case 2: encode_dispatch<2>(vec, (int)blocks, st, qp, x, n, ld, codes, ldc, zero_pad_to, norms, n_out); break;
    case 4: encode_dispatch<4>(vec, (int)blocks, st, qp, x, n, ld, codes, ldc, zero_pad_to, norms, n_out); break;
    case 8: encode_dispatch<8>(vec, (int)blocks, st, qp, x, n, ld, codes, ldc, zero_pad_to, norms, n_out); break;
    case 16: encode_dispatch<16>(vec, (int)blocks, st, qp, x, n, ld, codes, ldc, zero_pad_to, norms, n_out); break;
    case 32: encode_dispatch<32>(vec, (int)blocks, st, qp, x, n, ld, codes, ldc, zero_pad_to, norms, n_out); break;
    default: encode_dispatch<64>(vec, (int)blocks, st, qp, x, n, ld, codes, ldc, zero_pad_to, norms, n_out); break;
    }
    return hipGetLastError();
}

hipError_t launch_repack_i8(const int8_t *src, int64_t n, int64_t ld, int d, int8_t *dst, int64_t ldd,
                            int d_pad, int32_t *norms, hipStream_t st, int64_t n_out)
{
    if (n_out < n) n_out = n;
    if (n_out <= 0) return hipSuccess;
    const int64_t blocks = ceil_div(n_out * 16, 256);
    repack_i8_kernel<<<(unsigned)blocks, 256, 0, st>>>(src, n, ld, d, dst, ldd, d_pad, norms, n_out);
    return hipGetLastError();
}

hipError_t launch_pack4(const int8_t *src, int64_t n, int64_t ld, int d, uint8_t *dst, int d_pad, int32_t *norms,
                        hipStream_t st)
{
    if (n <= 0) return hipSuccess;
    pack4_kernel<<<(unsigned)ceil_div(n * 16, 256), 256, 0, st>>>(src, n, ld, d, dst, d_pad, norms);
    return hipGetLastError();
}

hipError_t launch_permute_queries(const int8_t *q, int64_t nq_pad, int d_pad, bool l2, int8_t *qperm, int32_t *qadj,
                                  hipStream_t st)
{
    if (nq_pad <= 0) return hipSuccess;
    permute_queries_kernel<<<(unsigned)ceil_div(nq_pad * 16, 256), 256, 0, st>>>(q, nq_pad, d_pad, l2 ? 1 : 0, qperm, qadj);
    return hipGetLastError();
}

hipError_t launch_zero_bytes(void *p, size_t bytes, hipStream_t st)
{
    const size_t words = bytes / 4;
    if (!words) return hipSuccess;
    size_t blocks = (words + 255) / 256;
    if (blocks > 1024) blocks = 1024;
    zero_words_kernel<<<(unsigned)blocks, 256, 0, st>>>((uint32_t *)p, words);
    return hipGetLastError();
}

hipError_t launch_item_aux(const int32_t *norms, int64_t row0, int64_t n_total, int32_t *cinit,
                           uint32_t *parity, hipStream_t st)
{
    const int64_t w0 = row0 / 32, w1 = ceil_div(n_total, 32);
    if (w1 <= w0) return hipSuccess;
    const int64_t blocks = ceil_div(w1 - w0, 256);
    item_aux_kernel<<<(unsigned)blocks, 256, 0, st>>>(norms, w0, w1, n_total, cinit, parity);
    return hipGetLastError();
}

}  // namespace lpq
