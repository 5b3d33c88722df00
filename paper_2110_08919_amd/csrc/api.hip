// C ABI of liblpq.so: argument checks, handle lifetimes, workspace planning and the order
// in which the kernels of a search are enqueued.  No kernel lives here.
#include <atomic>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <cmath>
#include <vector>

#include "lpq_internal.h"

using namespace lpq;

// ------------------------------------------------------------------------ errors ----
static thread_local char g_err[512] = "";

static int fail(int code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

#define HIP_TRY(expr)                                                                        \
    do {                                                                                     \
        hipError_t e_ = (expr);                                                              \
        if (e_ != hipSuccess)                                                                \
            return fail(e_ == hipErrorOutOfMemory ? LPQ_ENOMEM : LPQ_EDEVICE, "%s: %s", #expr, \
                        hipGetErrorString(e_));                                              \
    } while (0)

extern "C" const char *lpq_last_error(void) { return g_err; }

// ------------------------------------------------------------------------ tuning ----
// Process-wide and read by every planning call: atomics, so that a thread changing a knob while
// others search is not a data race (a search still sees each knob at some moment of its planning;
// results never depend on them).
static std::atomic<int64_t> g_tune[LPQ_TUNE_COUNT_];
static inline int64_t tune(int key) { return g_tune[key].load(std::memory_order_relaxed); }

extern "C" int lpq_set_tuning(int key, int64_t value)
{
    if (key < 0 || key >= LPQ_TUNE_COUNT_) return fail(LPQ_EINVAL, "unknown tuning key %d", key);
#ifndef LPQ_ABLATION
    if (key == LPQ_TUNE_DRY_RUN && value != 0)
        return fail(LPQ_EINVAL, "LPQ_TUNE_DRY_RUN exists only in builds compiled with -DLPQ_ABLATION");
#endif
    g_tune[key].store(value, std::memory_order_relaxed);
    return LPQ_OK;
}

// --------------------------------------------------------------------- profiling ----
namespace {
// Event pairs are created when profiling is switched on, not inside the searches they time: a
// span only takes the next free pair (spans beyond the pool go untimed and are counted as dropped).
constexpr size_t PROFILE_POOL = 4096;
struct Profile {
    std::mutex mu;
    bool on = false;
    struct Span { hipEvent_t a, b; int kind; };
    std::vector<Span> pool;    // pairs created by lpq_profile_enable(1)
    size_t used = 0;           // pairs handed out so far
    int64_t dropped = 0;
    void clear()
    {
        for (auto &s : pool) { (void)hipEventDestroy(s.a); (void)hipEventDestroy(s.b); }
        pool.clear();
        used = 0;
        dropped = 0;
    }
};
Profile g_prof;

struct KernelSpan {  // brackets one kernel launch with two events while profiling is on
    hipEvent_t a = nullptr, b = nullptr;
    hipStream_t st;
    explicit KernelSpan(hipStream_t s, int kind_ = LPQ_PROFILE_SCAN) : st(s)
    {
        std::lock_guard<std::mutex> l(g_prof.mu);
        if (!g_prof.on) return;
        if (g_prof.used >= g_prof.pool.size()) { ++g_prof.dropped; return; }
        Profile::Span &sp = g_prof.pool[g_prof.used++];
        sp.kind = kind_;
        a = sp.a; b = sp.b;
        (void)hipEventRecord(a, st);
    }
    ~KernelSpan()
    {
        if (a) (void)hipEventRecord(b, st);
    }
};
}  // namespace

extern "C" int lpq_profile_enable(int on)
{
    std::lock_guard<std::mutex> l(g_prof.mu);
    g_prof.clear();
    g_prof.on = false;
    if (on) {
        g_prof.pool.reserve(PROFILE_POOL);
        for (size_t i = 0; i < PROFILE_POOL; ++i) {
            Profile::Span sp = {nullptr, nullptr, 0};
            hipError_t e = hipEventCreate(&sp.a);
            if (e == hipSuccess) e = hipEventCreate(&sp.b);
            if (e != hipSuccess) {
                if (sp.a) (void)hipEventDestroy(sp.a);
                g_prof.clear();
                return fail(LPQ_EDEVICE, "hipEventCreate: %s", hipGetErrorString(e));
            }
            g_prof.pool.push_back(sp);
        }
        g_prof.on = true;
    }
    return LPQ_OK;
}

static int profile_sum(int kind, int64_t *launches, double *total_ms)
{
    if (!launches || !total_ms) return fail(LPQ_EINVAL, "null output");
    std::lock_guard<std::mutex> l(g_prof.mu);
    double tot = 0.0;
    int64_t cnt = 0;
    for (size_t i = 0; i < g_prof.used; ++i) {
        const Profile::Span &s = g_prof.pool[i];
        if (kind >= 0 && s.kind != kind) continue;
        HIP_TRY(hipEventSynchronize(s.b));
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, s.a, s.b));
        tot += ms;
        ++cnt;
    }
    *launches = cnt;
    *total_ms = tot;
    return LPQ_OK;
}

extern "C" int lpq_profile_read(int64_t *launches, double *total_ms) { return profile_sum(-1, launches, total_ms); }

extern "C" int lpq_profile_read_kind(int kind, int64_t *launches, double *total_ms)
{
    if (kind != LPQ_PROFILE_SCAN && kind != LPQ_PROFILE_SEED) return fail(LPQ_EINVAL, "unknown kernel kind %d", kind);
    return profile_sum(kind, launches, total_ms);
}

// ------------------------------------------------------------------------ probes ----
extern "C" int lpq_probe_mfma_i8(const void *operands_dev, size_t operand_bytes, int iters, double *tops, void *stream)
{
    if (!tops) return fail(LPQ_EINVAL, "null output");
    if (iters < 1 || iters > 10000000) return fail(LPQ_EINVAL, "iters = %d outside 1..10 000 000", iters);
    if (operands_dev && operand_bytes < 16) return fail(LPQ_EINVAL, "operand buffer smaller than 16 bytes");
    if (operands_dev && (uintptr_t)operands_dev % 16) return fail(LPQ_EINVAL, "operand buffer must be 16-byte aligned");
    *tops = 0.0;
    HIP_TRY(probe_mfma(operands_dev, operand_bytes, iters, tops, (hipStream_t)stream));
    return LPQ_OK;
}

extern "C" int lpq_probe_scan_core(const void *operands_dev, size_t operand_bytes, int stages, double *tops, void *stream)
{
    if (!tops) return fail(LPQ_EINVAL, "null output");
    if (stages < 1 || stages > 10000000) return fail(LPQ_EINVAL, "stages = %d outside 1..10 000 000", stages);
    if (operands_dev && operand_bytes < 16) return fail(LPQ_EINVAL, "operand buffer smaller than 16 bytes");
    if (operands_dev && (uintptr_t)operands_dev % 16) return fail(LPQ_EINVAL, "operand buffer must be 16-byte aligned");
    *tops = 0.0;
    HIP_TRY(probe_scan_core(operands_dev, operand_bytes, stages, tops, (hipStream_t)stream));
    return LPQ_OK;
}

extern "C" int lpq_probe_stream(const void *src_dev, size_t bytes, int mode, int reps, double *gbps, void *stream)
{
    if (!src_dev || !gbps) return fail(LPQ_EINVAL, "null argument");
    if (mode != 0 && mode != 1) return fail(LPQ_EINVAL, "unknown mode %d", mode);
    if (bytes < 4096 || reps < 1 || reps > 10000) return fail(LPQ_EINVAL, "bytes < 4096 or reps outside 1..10 000");
    if ((uintptr_t)src_dev % 16) return fail(LPQ_EINVAL, "buffer must be 16-byte aligned");
    *gbps = 0.0;
    HIP_TRY(probe_stream(src_dev, bytes / 4096 * 4096, mode, reps, gbps, (hipStream_t)stream));
    return LPQ_OK;
}

// --------------------------------------------------------------------- quantizer ----
struct lpq_quantizer {
    int d = 0, bits = 0;
    bool ready = false;
    float *params = nullptr;   // device [4][d]: k, S_b, S_e, m
    float *staging = nullptr;  // device [4][d]: calibration result before it is committed
    void *scratch = nullptr;   // calibration partials
    int *flag = nullptr;       // device: non-finite value seen
};

static QuantParams view(const float *params, int d, int bits)
{
    QuantParams qp;
    qp.k = params; qp.sb = params + d; qp.se = params + 2 * d; qp.m = params + 3 * d;
    qp.d = d; qp.bits = bits;
    return qp;
}

extern "C" void lpq_quantizer_destroy(lpq_quantizer *q)
{
    if (!q) return;
    (void)hipFree(q->params);
    (void)hipFree(q->staging);
    (void)hipFree(q->scratch);
    (void)hipFree(q->flag);
    delete q;
}

extern "C" int lpq_quantizer_create(lpq_quantizer **out, int d, int bits)
{
    if (!out) return fail(LPQ_EINVAL, "out is null");
    if (d < 1) return fail(LPQ_EINVAL, "d = %d < 1", d);
    if (bits < 1 || bits > 8) return fail(LPQ_EINVAL, "bits = %d outside 1..8", bits);
    if (d > MAX_D) return fail(LPQ_ERANGE, "d = %d > %d", d, (int)MAX_D);
    lpq_quantizer *q = new (std::nothrow) lpq_quantizer;
    if (!q) return fail(LPQ_ENOMEM, "host allocation failed");
    q->d = d; q->bits = bits;
    hipError_t e = hipMalloc(&q->params, sizeof(float) * 4 * d);
    if (e == hipSuccess) e = hipMalloc(&q->staging, sizeof(float) * 4 * d);
    if (e == hipSuccess) e = hipMalloc(&q->scratch, calib_scratch_bytes(d));
    if (e == hipSuccess) e = hipMalloc(&q->flag, 256);
    if (e != hipSuccess) {
        lpq_quantizer_destroy(q);
        return fail(e == hipErrorOutOfMemory ? LPQ_ENOMEM : LPQ_EDEVICE, "hipMalloc: %s", hipGetErrorString(e));
    }
    *out = q;
    return LPQ_OK;
}

extern "C" int lpq_quantizer_calibrate(lpq_quantizer *q, const float *x_dev, int64_t n, int64_t ld, int mode,
                                       int scope, float sigma_mult, void *stream)
{
    if (!q || !x_dev) return fail(LPQ_EINVAL, "null argument");
    if (n < 1) return fail(LPQ_EINVAL, "n = %lld < 1", (long long)n);
    if (ld < q->d) return fail(LPQ_EINVAL, "ld = %lld < d = %d", (long long)ld, q->d);
    if (mode < LPQ_CALIB_MINMAX || mode > LPQ_CALIB_QUANTILE) return fail(LPQ_EINVAL, "unknown calibration mode %d", mode);
    if (mode == LPQ_CALIB_QUANTILE && !(sigma_mult >= 0.0f && sigma_mult < 0.5f)) return fail(LPQ_EINVAL, "clip fraction must be in [0, 0.5)");
    if (scope != LPQ_SCOPE_PER_FEATURE && scope != LPQ_SCOPE_GLOBAL && scope != LPQ_SCOPE_SHARED_WIDTH) return fail(LPQ_EINVAL, "unknown scope %d", scope);
    if (mode == LPQ_CALIB_GAUSS && !(sigma_mult > 0.0f)) return fail(LPQ_EINVAL, "sigma_mult must be > 0");
    hipStream_t st = (hipStream_t)stream;
    HIP_TRY(launch_calibrate(x_dev, n, ld, q->d, q->bits, mode, scope, (double)sigma_mult, q->scratch,
                             q->staging, q->flag, st));
    int bad = 0;
    HIP_TRY(hipMemcpyAsync(&bad, q->flag, sizeof(int), hipMemcpyDeviceToHost, st));
    HIP_TRY(hipStreamSynchronize(st));
    if (bad) return fail(LPQ_ENONFINITE, "calibration data holds a NaN or an infinity");
    HIP_TRY(hipMemcpyAsync(q->params, q->staging, sizeof(float) * 4 * q->d, hipMemcpyDeviceToDevice, st));
    HIP_TRY(hipStreamSynchronize(st));
    q->ready = true;
    return LPQ_OK;
}

extern "C" int lpq_quantizer_set_params(lpq_quantizer *q, const float *k, const float *s_b, const float *s_e)
{
    if (!q || !k || !s_b || !s_e) return fail(LPQ_EINVAL, "null argument");
    const size_t bytes = sizeof(float) * q->d;
    HIP_TRY(hipMemcpy(q->params, k, bytes, hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(q->params + q->d, s_b, bytes, hipMemcpyHostToDevice));
    HIP_TRY(hipMemcpy(q->params + 2 * q->d, s_e, bytes, hipMemcpyHostToDevice));
    HIP_TRY(launch_derive_m(q->params, q->d, q->bits, nullptr));
    HIP_TRY(hipDeviceSynchronize());
    q->ready = true;
    return LPQ_OK;
}

extern "C" int lpq_quantizer_get_params(const lpq_quantizer *q, float *k, float *s_b, float *s_e, float *m)
{
    if (!q || !k || !s_b || !s_e) return fail(LPQ_EINVAL, "null argument");
    if (!q->ready) return fail(LPQ_ESTATE, "quantizer has no constants yet");
    const size_t bytes = sizeof(float) * q->d;
    HIP_TRY(hipDeviceSynchronize());
    HIP_TRY(hipMemcpy(k, q->params, bytes, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(s_b, q->params + q->d, bytes, hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(s_e, q->params + 2 * q->d, bytes, hipMemcpyDeviceToHost));
    if (m) HIP_TRY(hipMemcpy(m, q->params + 3 * q->d, bytes, hipMemcpyDeviceToHost));
    return LPQ_OK;
}

extern "C" int lpq_encode(const lpq_quantizer *q, const float *x_dev, int64_t n, int64_t ld, int8_t *codes_dev,
                          int64_t ld_codes, int32_t *norms_dev, void *stream)
{
    if (!q || !x_dev || !codes_dev) return fail(LPQ_EINVAL, "null argument");
    if (n < 0) return fail(LPQ_EINVAL, "n < 0");
    if (ld < q->d || ld_codes < q->d) return fail(LPQ_EINVAL, "row stride smaller than d = %d", q->d);
    if (!q->ready) return fail(LPQ_ESTATE, "encode before calibrate/set_params");
    HIP_TRY(launch_encode(view(q->params, q->d, q->bits), x_dev, n, ld, codes_dev, ld_codes, 0, norms_dev,
                          (hipStream_t)stream));
    return LPQ_OK;
}

// ------------------------------------------------------------------------- index ----
struct lpq_index {
    int d = 0, d_pad = 0, bits = 0;
    bool packed = false;         // two 4-bit codes per byte: rows of d_pad / 2 bytes
    int64_t capacity = 0, cap_rows = 0, size = 0;
    float *params = nullptr;     // device copy of the quantizer constants
    int8_t *codes = nullptr;     // [cap_rows][d_pad], zero padded
    int32_t *norms = nullptr;    // [cap_rows]
    int32_t *cinit = nullptr;    // [cap_rows]   accumulator seeds of the matrix-core kernel
    uint32_t *parity = nullptr;  // [cap_rows/32]
    int8_t *stage = nullptr;     // packed only: [PACK_STAGE_ROWS][d_pad] int8 codes on their way to nibbles
};
constexpr int64_t PACK_STAGE_ROWS = 65536;

extern "C" void lpq_index_destroy(lpq_index *idx)
{
    if (!idx) return;
    (void)hipFree(idx->params);
    (void)hipFree(idx->codes);
    (void)hipFree(idx->norms);
    (void)hipFree(idx->cinit);
    (void)hipFree(idx->stage);
    (void)hipFree(idx->parity);
    delete idx;
}

// Row length an index stores d features in: a length the matrix-core scans have where one exists.
static int padded_row_length(int d)
{
    // up to 1536 features: the row lengths the matrix-core kernels take; beyond: the generic kernel's
    return d <= 64 ? 64 : d <= 96 ? 96 : d <= 128 ? 128 : d <= 192 ? 192 : d <= 256 ? 256
           : d <= 384 ? 384 : d <= 512 ? 512 : d <= 768 ? 768 : d <= 1024 ? 1024 : d <= 1536 ? 1536 : (int)round_up(d, 32);
}

static int index_create_impl(lpq_index **out, const lpq_quantizer *q, int64_t capacity, bool packed)
{
    if (!out || !q) return fail(LPQ_EINVAL, "null argument");
    if (!q->ready) return fail(LPQ_ESTATE, "quantizer has no constants yet");
    if (packed && q->bits > 4) return fail(LPQ_EINVAL, "packed storage needs a quantizer of at most 4 bits (has %d)", q->bits);
    if (packed && q->d > MAX_D_PACKED)
        return fail(LPQ_ERANGE, "packed storage is searched for at most %d features (has %d)", (int)MAX_D_PACKED, q->d);
    if (capacity < 1) return fail(LPQ_EINVAL, "capacity < 1");
    if (capacity >= (int64_t(1) << 31) - 1024) return fail(LPQ_ERANGE, "capacity must stay below 2^31 - 1024");
    lpq_index *idx = new (std::nothrow) lpq_index;
    if (!idx) return fail(LPQ_ENOMEM, "host allocation failed");
    idx->d = q->d; idx->bits = q->bits;
    idx->packed = packed;
    // Rows are zero padded to a length the matrix-core scans have (64, 96, 128, 192 or 256 bytes):
    // up to 256 features never fall back to the generic kernel, which is ~100x slower on large
    // batches; the price is up to 2x the row bytes for d <= 32 and 20 % for 129..160.
    idx->d_pad = padded_row_length(q->d);
    idx->capacity = capacity;
    idx->cap_rows = round_up(capacity, 256) + 256;  // whole tiles may be read past the last item
    const size_t code_bytes = (size_t)idx->cap_rows * idx->d_pad / (packed ? 2 : 1);
    hipError_t e = hipMalloc(&idx->params, sizeof(float) * 4 * idx->d);
    if (e == hipSuccess) e = hipMalloc(&idx->codes, code_bytes);
    if (e == hipSuccess && packed) e = hipMalloc(&idx->stage, (size_t)PACK_STAGE_ROWS * idx->d_pad);
    if (e == hipSuccess) e = hipMalloc(&idx->norms, sizeof(int32_t) * idx->cap_rows);
    if (e == hipSuccess) e = hipMalloc(&idx->cinit, sizeof(int32_t) * idx->cap_rows);
    if (e == hipSuccess) e = hipMalloc(&idx->parity, sizeof(uint32_t) * (idx->cap_rows / 32));
    if (e == hipSuccess) e = hipMemcpy(idx->params, q->params, sizeof(float) * 4 * idx->d, hipMemcpyDeviceToDevice);
    if (e == hipSuccess) e = hipMemset(idx->codes, packed ? 0x88 : 0, code_bytes);   // code 0 everywhere
    if (e == hipSuccess) e = hipMemset(idx->norms, 0, sizeof(int32_t) * idx->cap_rows);
    if (e == hipSuccess) e = hipMemset(idx->parity, 0, sizeof(uint32_t) * (idx->cap_rows / 32));
    if (e == hipSuccess) e = hipMemsetD32((hipDeviceptr_t)idx->cinit, CINIT_PAD, (size_t)idx->cap_rows);
    if (e == hipSuccess) e = hipDeviceSynchronize();
    if (e != hipSuccess) {
        lpq_index_destroy(idx);
        return fail(e == hipErrorOutOfMemory ? LPQ_ENOMEM : LPQ_EDEVICE, "index allocation: %s", hipGetErrorString(e));
    }
    *out = idx;
    return LPQ_OK;
}

extern "C" int lpq_index_create(lpq_index **out, const lpq_quantizer *q, int64_t capacity)
{
    return index_create_impl(out, q, capacity, false);
}

extern "C" int lpq_index_create_packed(lpq_index **out, const lpq_quantizer *q, int64_t capacity)
{
    return index_create_impl(out, q, capacity, true);
}

// Packed index: rows [row0, row0 + n) from int8 codes (device), through the nibble packer.
static int index_pack_rows(lpq_index *idx, int64_t row0, const int8_t *codes, int64_t n, int64_t ld, hipStream_t st)
{
    HIP_TRY(launch_pack4(codes, n, ld, idx->d, reinterpret_cast<uint8_t *>(idx->codes) + (size_t)row0 * (idx->d_pad / 2),
                         idx->d_pad, idx->norms + row0, st));
    return LPQ_OK;
}

static int index_after_add(lpq_index *idx, int64_t n, hipStream_t st)
{
    const int64_t row0 = idx->size;
    idx->size += n;
    // Seeds for every row of every tile that can be touched: rows beyond size get the padding seed.
    HIP_TRY(launch_item_aux(idx->norms, row0, idx->size, idx->cinit, idx->parity, st));
    return LPQ_OK;
}

extern "C" int lpq_index_add_f32(lpq_index *idx, const float *x_dev, int64_t n, int64_t ld, void *stream)
{
    if (!idx || !x_dev) return fail(LPQ_EINVAL, "null argument");
    if (n < 0) return fail(LPQ_EINVAL, "n < 0");
    if (ld < idx->d) return fail(LPQ_EINVAL, "ld < d");
    if (idx->size + n > idx->capacity) return fail(LPQ_ERANGE, "index capacity %lld exceeded", (long long)idx->capacity);
    if (n == 0) return LPQ_OK;
    hipStream_t st = (hipStream_t)stream;
    if (idx->packed) {   // encode a chunk into the staging rows, pack it, next chunk
        for (int64_t r = 0; r < n; r += PACK_STAGE_ROWS) {
            const int64_t m = n - r < PACK_STAGE_ROWS ? n - r : PACK_STAGE_ROWS;
            HIP_TRY(launch_encode(view(idx->params, idx->d, idx->bits), x_dev + r * ld, m, ld, idx->stage, idx->d_pad,
                                  idx->d_pad, nullptr, st));
            const int rc = index_pack_rows(idx, idx->size + r, idx->stage, m, idx->d_pad, st);
            if (rc) return rc;
        }
        return index_after_add(idx, n, st);
    }
    HIP_TRY(launch_encode(view(idx->params, idx->d, idx->bits), x_dev, n, ld,
                          idx->codes + (size_t)idx->size * idx->d_pad, idx->d_pad, idx->d_pad,
                          idx->norms + idx->size, st));
    return index_after_add(idx, n, st);
}

extern "C" int lpq_index_add_i8(lpq_index *idx, const int8_t *codes_dev, int64_t n, int64_t ld, void *stream)
{
    if (!idx || !codes_dev) return fail(LPQ_EINVAL, "null argument");
    if (n < 0) return fail(LPQ_EINVAL, "n < 0");
    if (ld < idx->d) return fail(LPQ_EINVAL, "ld < d");
    if (idx->size + n > idx->capacity) return fail(LPQ_ERANGE, "index capacity %lld exceeded", (long long)idx->capacity);
    if (n == 0) return LPQ_OK;
    hipStream_t st = (hipStream_t)stream;
    if (idx->packed) {
        const int rc = index_pack_rows(idx, idx->size, codes_dev, n, ld, st);
        return rc ? rc : index_after_add(idx, n, st);
    }
    HIP_TRY(launch_repack_i8(codes_dev, n, ld, idx->d, idx->codes + (size_t)idx->size * idx->d_pad, idx->d_pad,
                             idx->d_pad, idx->norms + idx->size, st));
    return index_after_add(idx, n, st);
}

extern "C" int64_t lpq_index_size(const lpq_index *idx) { return idx ? idx->size : -1; }

extern "C" int lpq_index_data(const lpq_index *idx, const int8_t **codes_dev, int64_t *ld_codes,
                              const int32_t **norms_dev)
{
    if (!idx) return fail(LPQ_EINVAL, "null index");
    if (codes_dev) *codes_dev = idx->codes;
    if (ld_codes) *ld_codes = idx->packed ? idx->d_pad / 2 : idx->d_pad;
    if (norms_dev) *norms_dev = idx->norms;
    return LPQ_OK;
}

// -------------------------------------------------------------- candidate lists ----
extern "C" int lpq_gather_dist_i8(const lpq_index *idx, const int8_t *qcodes_dev, int64_t nq, int64_t ld,
                                  const int32_t *ids_dev, int m, int metric, int32_t *dist_dev, void *stream)
{
    if (!idx) return fail(LPQ_EINVAL, "null index");
    if (nq < 0 || m < 1) return fail(LPQ_EINVAL, "nq < 0 or m < 1");
    if (metric != LPQ_METRIC_L2SQ && metric != LPQ_METRIC_IP) return fail(LPQ_EINVAL, "unknown metric %d", metric);
    if (idx->size < 1) return fail(LPQ_ESTATE, "gather on an empty index");
    if (nq > 0 && (!qcodes_dev || !ids_dev || !dist_dev)) return fail(LPQ_EINVAL, "null argument");
    if (nq > 0 && ld < idx->d) return fail(LPQ_EINVAL, "ld < d");
    HIP_TRY(launch_gather_dist(idx->codes, idx->norms, idx->size, idx->d, idx->d_pad, qcodes_dev, nq, ld, ids_dev, m,
                               metric, dist_dev, (hipStream_t)stream, idx->packed));
    return LPQ_OK;
}

extern "C" int lpq_rerank_f32(const float *x_dev, int64_t n, int64_t ldx, const float *q_dev, int64_t nq, int64_t ldq,
                              int d, const int32_t *cand_ids_dev, int kc, int k, int metric, int32_t *ids_dev,
                              float *dist_dev, void *stream)
{
    if (d < 1 || n < 1 || nq < 0 || kc < 1 || k < 1) return fail(LPQ_EINVAL, "bad size");
    if (metric != LPQ_METRIC_L2SQ && metric != LPQ_METRIC_IP) return fail(LPQ_EINVAL, "unknown metric %d", metric);
    if (kc > 4096) return fail(LPQ_ERANGE, "kc = %d > 4096", kc);
    if (k > 4096) return fail(LPQ_ERANGE, "k = %d > 4096", k);
    if (ldx < d || (nq > 0 && ldq < d)) return fail(LPQ_EINVAL, "row stride < d");
    if (!x_dev || (nq > 0 && (!q_dev || !cand_ids_dev || !ids_dev || !dist_dev))) return fail(LPQ_EINVAL, "null argument");
    HIP_TRY(launch_rerank_f32(x_dev, n, ldx, q_dev, nq, ldq, d, cand_ids_dev, kc, k, metric, ids_dev, dist_dev,
                              (hipStream_t)stream));
    return LPQ_OK;
}

// ------------------------------------------------------------------------ search ----
namespace {

// How a search over n items is cut up, and where its intermediates live in the workspace.
enum PlanMode { PLAN_GENERIC = 0, PLAN_MFMA_LDS = 1, PLAN_MFMA_REG = 2, PLAN_MFMA_COLLECT = 3 };
struct Plan {
    int mode = PLAN_GENERIC;
    int64_t nq_pad = 0;
    int64_t seed_rows = 0;  // rows of the threshold-seeding pass (0 = none)
    int S1 = 0, S2 = 0;     // corpus splits of the seeding pass and of the main pass
    int SEG = 0;            // PLAN_MFMA_REG: segments per split in the seeding pass
    int G = 0;              // PLAN_MFMA_REG: group maxima per query
    bool rsplit = false;    // PLAN_MFMA_REG, PLAN_MFMA_COLLECT: row-split workgroups (few queries)
    int rs_waves = 0;       // ... of this many waves (0 when not row-split)
    int merge_group = 0;    // lists merged per workgroup in the first merge pass (0 = single pass)
    int64_t seed_stride = 0;   // seeding pass: one stage every seed_stride rows (systematic sample)
    int seed_stages = 0;       // ... seed_stages of them per split
    int64_t piece_stride = 0;  // seeding pass: or runs of 8 rows every piece_stride rows, dealt round-robin to the splits
    int piece_stages = 0;      // ... eight runs to a stage, piece_stages stages per split
    int SS = 0, Cs = 0;     // PLAN_MFMA_COLLECT: regions per query, capacity of a region
    int Sg = 0;             // PLAN_MFMA_COLLECT: splits of the generic kernel for overflowed queries
    int Sr = 0;             // PLAN_MFMA_COLLECT: splits of the register-list kernel for many overflowed queries (0 = none)
    int rounds = 0;         // PLAN_MFMA_COLLECT: further rounds of the collecting scan, with tighter bounds, for overflowed queries
    int wave_queries = 64;  // PLAN_MFMA_COLLECT: queries per wave of the scan
    int expect = 0;         // PLAN_MFMA_COLLECT: expected candidates per query
    size_t off_qcodes = 0, off_qnorms = 0, off_lists1 = 0, off_seedlist = 0, off_seeds = 0, off_lists2 = 0,
           off_gmax = 0, off_merge_tmp = 0, off_cbuf = 0, off_ccnt = 0, off_over = 0, off_qlist = 0, off_redo = 0, off_bounds2 = 0, off_over2 = 0,
           off_qlist2 = 0, total = 0;
};

size_t align256(size_t v) { return (v + 255) & ~size_t(255); }

constexpr int WIDE_MIN_BITS = 2;
constexpr int64_t PACKED_BATCH_MIN = 128;  // packed index: larger batches take one collecting scan instead of tiles of 64 queries
constexpr int REFINE_ROUNDS = 2;        // further rounds of the collecting scan for queries that overflowed (k > 16)
constexpr int REFINE_GENERIC_MAX = 16;  // ... unless the first round flags no more than this many (generic kernel then)   // narrowest codes that take the 128-queries-per-wave collecting scan

Plan make_plan(const lpq_index *idx, int64_t nq, int k)
{
    Plan p;
    const int64_t n = idx->size;
    const int64_t want = tune(LPQ_TUNE_PATH);
    const bool regs = mfma_reg_supported(idx->d_pad, k), coll = mfma_collect_supported(idx->d_pad, k);
    // Large batches of short rows: the collecting variant with 128 queries per wave beats the
    // register lists at any k it takes (fewer LDS reads and less per-stage overhead per contraction).
    // (Not for codes of fewer than WIDE_MIN_BITS bits: there many items tie at the seed
    // threshold, all of them are collected, and queries spill to the exact redo.)
    const bool wide = coll && idx->bits >= WIDE_MIN_BITS && mfma_collect_wide(nq, idx->d_pad) &&
                      tune(LPQ_TUNE_WAVE_QUERIES) != 64;
    // Rows longer than 128 bytes: the register-list kernels hold 6 or 8 operand registers per query
    // block on top of the lists and spill; the collecting variant measured 1.6x (10 000 queries) to
    // 3.5x (16 queries) faster at d = 256 for every batch size and code width.
    const bool long_rows = coll && idx->d_pad > 128;
    // Lists of 11 to 16 entries: the 16-entry register lists cost more per accepted candidate than
    // collecting does; collecting measured 11 to 40 % faster at every batch size (d = 64 to 128).
    const bool long_lists = coll && k > 10;
    // Packed rows: the row-split register-list kernel (callers tile the queries by 64), or for large
    // batches the collecting scan over all queries at once; the generic kernel on request.
    // (lists of more than 16 entries: the collecting scan at every batch size; rows of 32 packed
    // bytes have no scan over more than 64 queries, their callers tile)
    const bool packed_batch = idx->packed && coll && idx->d_pad >= 96 && (nq > PACKED_BATCH_MIN || (!regs && nq > 64));
    const bool packed_collect = packed_batch || (idx->packed && coll && !regs && nq <= 64);
    if (idx->packed) p.mode = want == 1 ? PLAN_GENERIC : (packed_collect ? PLAN_MFMA_COLLECT
                                                          : (regs ? PLAN_MFMA_REG : PLAN_GENERIC));
    else if (want == 3 && coll) p.mode = PLAN_MFMA_COLLECT;
    else if (want != 1 && want != 4 && (wide || long_rows || long_lists)) p.mode = PLAN_MFMA_COLLECT;
    else if (want != 1 && regs) p.mode = PLAN_MFMA_REG;
    else if (want != 1 && want != 4 && coll) p.mode = PLAN_MFMA_COLLECT;
    else if (want != 1 && mfma_lds_supported(idx->d_pad, k)) p.mode = PLAN_MFMA_LDS;
    // Corpora too small for any sample (below 4096 rows) and little work in all: the generic kernel
    // (1000 x 128, 1000 queries, k = 10: 0.05 ms against 0.29 ms for an unseeded matrix-core scan).
    if (want == 0 && n < 4096 && nq * n <= (int64_t(4) << 20)) p.mode = PLAN_GENERIC;
    p.nq_pad = round_up(nq > 0 ? nq : 1, 512);
    // A merge pass sorts up to 4096 candidates per workgroup; more lists than that are merged in
    // two passes, so the number of splits is bounded by max_lists^2 only.
    const int max_lists = merge_max_lists(k) * (merge_max_lists(k) > 1 ? merge_max_lists(k) : 1);
    const int64_t slots = 512;   // workgroups of the matrix-core kernels resident at once (2 per CU)

    // Seeding pass over a sample of the corpus: it yields, per query, an upper bound on the final
    // k-th best key, so the main pass rejects almost everything from its first tile on.
    // PLAN_MFMA_REG and PLAN_MFMA_COLLECT derive the bound from group maxima over chunks spread
    // evenly over the corpus (no candidates collected) and then scan ALL rows; PLAN_MFMA_LDS
    // searches a first slice exactly and scans the rest.  The collecting scan never tightens the
    // bound, so its sample is a fixed fraction of the corpus: about k n / seed_rows candidates
    // per query survive.
    const bool gm = p.mode == PLAN_MFMA_REG || p.mode == PLAN_MFMA_COLLECT;
    int64_t seed = 0;
    if (tune(LPQ_TUNE_SEED_ROWS) > 0) seed = tune(LPQ_TUNE_SEED_ROWS);
    else if (tune(LPQ_TUNE_SEED_ROWS) == 0 && p.mode != PLAN_GENERIC) {
        // Few queries: the scan is bound by corpus bytes, so the sample stays small.  Otherwise a
        // larger sample pays for itself through fewer candidates in the main pass (measured).
        const bool few = gm && mfma_row_split(nq, idx->d_pad, idx->packed);
        seed = gm ? (few ? n / 16 : n / 8) : n / 64;
        // (corpora below 64K rows: the sample may go down to 1024 rows - without a seeding pass every
        // split spends its few hundred rows filling lists from empty thresholds: 10 000 x 128, 100
        // queries: 0.245 ms unseeded)
        const int64_t lo_gm = n >= 65536 ? 8192 : (n / 8 > 1024 ? n / 8 : 1024);
        const int64_t lo = gm ? lo_gm : 4096, hi = p.mode == PLAN_MFMA_COLLECT ? n : (gm ? (few ? 65536 : 131072) : 32768);
        seed = seed < lo ? lo : (seed > hi ? hi : seed);
        if (p.mode == PLAN_MFMA_COLLECT && few) {   // no tightening during the scan: the sample grows with k
            // (beyond k = 256 a quarter: an eighth would let about 9 k candidates through, more than the
            // 4096 the selection sorts)
            const int64_t by_k = n / 400 * k, least = n / 16, most = k > 512 ? n / 2 : (k > 256 ? n / 4 : n / 8);
            seed = by_k < least ? least : (by_k > most ? most : by_k);
        } else if (p.mode == PLAN_MFMA_COLLECT) {
            // The sample costs time in proportion to its rows, the candidates it lets through in
            // proportion to k n / rows: the sum is least at rows ~ sqrt(k n) (coefficient measured:
            // 125 000 rows at n = 1M, k = 10).  At least k n / 1500, so that the ~1.15 k n / rows
            // candidates of a query stay well inside the 4096 the selection kernel sorts; at most n / 4.
            const double by_cost = 125000.0 * std::sqrt((double)n / 1e6 * (double)k / 10.0);
            const double by_room = (double)k * (double)n / 1500.0;
            const double want_rows = by_cost > by_room ? by_cost : by_room;
            // (k beyond 512: half the corpus, or the ~4.6 k candidates a quarter lets through would not fit)
            const int64_t most = k > 512 ? n / 2 : n / 4;
            seed = want_rows > (double)most ? most : (int64_t)want_rows;
        }
    }
    seed = seed / 256 * 256;
    // A sample must hold at least 64 k rows for its k-th group maximum to mean something; a small
    // corpus may give up to half of its rows for that (20 000 x 128, 10 000 queries, k = 100: 0.5 ms
    // with such a sample against 2.3 ms through the generic kernel).
    if (p.mode == PLAN_MFMA_COLLECT && seed > 0 && seed < 64 * (int64_t)k) seed = round_up(64 * (int64_t)k, 256);
    if (seed < 64 * k || seed * 2 > n || (k <= 512 && p.mode != PLAN_MFMA_COLLECT && seed * 4 > n)) seed = 0;
    if (p.mode == PLAN_MFMA_COLLECT && !seed) {   // too few items to sample: exact paths
        // (longer lists without a sample: the generic kernel; the LDS-list matrix-core kernel measured
        // 10 to 70x slower on the corpora this happens for - 1000 x 128, k = 100, 1000 queries: 4.3 ms
        // against 0.06 ms - and stays reachable through LPQ_TUNE_PATH = 4)
        p.mode = (regs && want != 1) ? PLAN_MFMA_REG
                 : (want == 4 && mfma_lds_supported(idx->d_pad, k) && !idx->packed ? PLAN_MFMA_LDS : PLAN_GENERIC);
    }

    // lists one merge launch takes: the register-list scan's come out sorted, which allows more of them
    const int one_pass = p.mode == PLAN_MFMA_REG ? merge_max_sorted_lists(k) : merge_max_lists(k);
    auto splits_for = [&](int64_t rows, int64_t tiles_q, int64_t min_rows, int64_t slots, int64_t cap) {
        int64_t s;
        if (p.mode != PLAN_GENERIC) s = tune(LPQ_TUNE_SPLITS) > 0 ? tune(LPQ_TUNE_SPLITS) : slots / (tiles_q > 0 ? tiles_q : 1);
        else s = tune(LPQ_TUNE_SPLITS) > 0 ? tune(LPQ_TUNE_SPLITS) : ceil_div(2048, nq > 0 ? nq : 1);
        const int64_t by_rows = rows / min_rows > 0 ? rows / min_rows : 1;
        if (s > by_rows) s = by_rows;
        if (s > cap) s = cap;
        if (s < 1) s = 1;
        return (int)s;
    };
    const bool gmode = p.mode == PLAN_MFMA_REG || p.mode == PLAN_MFMA_COLLECT;
    int64_t qt = (p.mode == PLAN_MFMA_LDS && k > 16) ? 128 : 256;   // queries per workgroup
    int64_t slots_now = slots;
    bool long_scan = false;
    if (gmode) {
        // (rows of more than 128 bytes: the collecting scan only - the register lists do not fit beside them)
        const int waves = mfma_row_split_waves(idx->d_pad, idx->packed);
        p.rsplit = mfma_row_split(nq, idx->d_pad, idx->packed) && (waves == 4 || p.mode == PLAN_MFMA_COLLECT);
        p.rs_waves = p.rsplit ? waves : 0;
        if (p.mode == PLAN_MFMA_COLLECT && mfma_collect_wide(nq, idx->d_pad) && tune(LPQ_TUNE_WAVE_QUERIES) != 64)
            p.wave_queries = 128;
        if (p.mode == PLAN_MFMA_COLLECT && idx->packed)   // the packed scan has one variant per row length
            p.wave_queries = idx->d_pad <= 128 ? 128 : 64;
        qt = mfma_queries_per_workgroup(nq, idx->d_pad, p.wave_queries == 128);
        long_scan = p.mode == PLAN_MFMA_COLLECT && !idx->packed && !p.rsplit && mfma_long_rows(idx->d_pad, nq);
        if (long_scan) {   // the scan for long rows and its seeding pass have their own tiles
            p.wave_queries = mfma_long_wave_queries(idx->d_pad);
            qt = (int64_t)mfma_long_waves(idx->d_pad, nq) * p.wave_queries;
            if (qt > 512) p.nq_pad = round_up(nq > 0 ? nq : 1, qt);   // query rows (codes, group maxima) cover whole tiles
            if (mfma_long_waves(idx->d_pad, nq) == 8) slots_now = 256;   // one workgroup per CU
        }
    }
    const int64_t tiles_q = ceil_div(nq > 0 ? nq : 1, qt);
    const int64_t min_rows = p.mode == PLAN_GENERIC ? 2048 : 512;
    if (seed) {
        // group maxima per query: 2 per split and segment (8 when rows are split), at most 2048 (4096 for k > 512)
        p.S1 = splits_for(seed, tiles_q, min_rows, slots_now, gmode ? (p.rsplit ? 256 : 1024) : merge_max_lists(k));
        if (gmode) {
            p.SEG = mfma_seed_segments(p.S1, k, p.rs_waves);
            p.G = mfma_seed_groups(p.S1, p.SEG, p.rs_waves);
            // systematic sample: one stage every seed_stride rows, shared out over the S1 splits
            const int64_t stage_rows = p.rsplit ? 32 * p.rs_waves : (long_scan ? mfma_long_stage_rows(idx->d_pad, nq) : 64);
            const int64_t stages = seed / stage_rows;
            p.seed_stages = (int)ceil_div(stages, p.S1);
            p.seed_stride = n / ((int64_t)p.seed_stages * p.S1) / 128 * 128;
            if (p.seed_stages < 1 || p.seed_stride < stage_rows) { p.seed_stages = 0; p.seed_stride = 0; }
            else seed = (int64_t)p.seed_stages * p.S1 * stage_rows;
            // Finer still (not for row-split launches): runs of 8 rows every piece_stride rows, dealt
            // round-robin to the splits, so that a run of neighbouring rows - a cluster stored
            // contiguously - is spread over many splits and hence over many groups of the pass.
            // (For k > 16 on a corpus sorted by norm a split's groups then span wide slices of the order
            // and up to a tenth of the queries overflow; the further rounds of the scan take those.)
            if (!p.rsplit && !long_scan) {
                const int64_t pstages = ceil_div(stages, p.S1);                 // as many rows as the stage-wise sample
                const int64_t pstride = pstages > 0 ? n / (8 * pstages * p.S1) : 0;   // all pieces inside the corpus
                if (pstride >= 16 && pstages >= 1) {
                    p.piece_stride = pstride;
                    p.piece_stages = (int)pstages;
                    seed = pstages * p.S1 * 64;
                }
            }
        }
    }
    p.seed_rows = seed;
    p.S2 = splits_for(gmode ? n : n - seed, tiles_q, min_rows, slots_now,
                      p.mode == PLAN_MFMA_COLLECT ? (p.rsplit ? 512 : 2048)
                                                  : (p.rsplit ? one_pass : max_lists));   // few queries: one merge pass
    if (p.mode == PLAN_MFMA_COLLECT) {
        // expected candidates per query ~ k n / seed_rows, spread evenly over SS regions (the scan
        // deals its stages round-robin to the splits); a region holds three times its share, at
        // least 64, which leaves room for bounds several times looser than expected (a corpus stored
        // in sorted order).  Overflow is caught per query and redone exactly.
        p.SS = mfma_collect_regions(p.S2, p.rs_waves);
        const double per_region = 1.15 * (double)k * (double)n / (double)seed / p.SS;
        p.expect = (int)(per_region * p.SS + 1.0);
        int64_t cs = 64;
        while ((double)cs < 3.0 * per_region && cs < 4096) cs <<= 1;
        p.Cs = (int)cs;
        if (tune(LPQ_TUNE_REGION_CAP) > 0) p.Cs = (int)(tune(LPQ_TUNE_REGION_CAP) < 4096 ? tune(LPQ_TUNE_REGION_CAP) : 4096);
        // splits of the redo scan: many, so that a few queries spread over the chip; bounded by the
        // single merge pass and by 256 MB of lists
        p.Sg = merge_max_lists(k) < 128 ? merge_max_lists(k) : 128;
        while (p.Sg > 4 && (size_t)nq * p.Sg * k * sizeof(cand_t) > (size_t(256) << 20)) p.Sg /= 2;
    }

    size_t o = 0;
    p.off_qcodes = o;   o = align256(o + (size_t)p.nq_pad * idx->d_pad);
    p.off_qnorms = o;   o = align256(o + (size_t)p.nq_pad * sizeof(int32_t));
    p.off_lists1 = o;   o = align256(o + (gmode ? 0 : (size_t)nq * p.S1 * k * sizeof(cand_t)));
    p.off_seedlist = o; o = align256(o + (size_t)nq * k * sizeof(cand_t));
    p.off_seeds = o;    o = align256(o + (size_t)p.nq_pad * sizeof(cand_t));
    p.off_lists2 = o;
    o = align256(o + (size_t)nq * (p.mode == PLAN_MFMA_COLLECT ? p.Sg : p.S2) * k * sizeof(cand_t));
    p.off_gmax = o;
    if (gmode && seed) o = align256(o + (size_t)p.nq_pad * p.G * sizeof(int32_t));
    p.off_merge_tmp = o;
    if (p.mode != PLAN_MFMA_COLLECT && p.S2 > one_pass) {
        p.merge_group = merge_max_lists(k);
        o = align256(o + (size_t)nq * ceil_div(p.S2, p.merge_group) * k * sizeof(cand_t));
    }
    if (p.mode == PLAN_MFMA_COLLECT) {
        p.off_cbuf = o; o = align256(o + (size_t)nq * p.SS * p.Cs * sizeof(cand_t));
        p.off_ccnt = o; o = align256(o + (size_t)nq * p.SS * sizeof(int32_t));
        p.off_over = o; o = align256(o + (size_t)nq * sizeof(int32_t));
        p.off_qlist = o; o = align256(o + ((size_t)nq + 1) * sizeof(int32_t));   // redo list, then its counter
        // redo of many queries by the register-list kernel (k <= 16, 256 queries per workgroup): one
        // list per query and split, few enough splits for a single merge pass
        if (!p.rsplit && regs && !idx->packed) {
            int64_t sr = slots / ceil_div(nq, 256);
            if (sr > merge_max_lists(k)) sr = merge_max_lists(k);
            if (sr > n / 512) sr = n / 512;
            p.Sr = (int)(sr < 1 ? 1 : sr);
            p.off_redo = o; o = align256(o + (size_t)nq * p.Sr * k * sizeof(cand_t));
        }
        // longer lists: a second collecting scan of the flagged queries, bounded by what the first collected
        if (!p.Sr) {
            p.rounds = p.rsplit ? 1 : REFINE_ROUNDS;   // few queries: every launch counts, and their many regions rarely overflow twice
            p.off_bounds2 = o; o = align256(o + (size_t)p.nq_pad * sizeof(cand_t));
            p.off_over2 = o;   o = align256(o + (size_t)p.rounds * nq * sizeof(int32_t));
            p.off_qlist2 = o;  o = align256(o + (size_t)p.rounds * (nq + 1) * sizeof(int32_t));   // per round: list, then its counter
        }
    }
    p.total = o;
    return p;
}

int check_search_args(const lpq_index *idx, const void *q, int64_t nq, int64_t ld, int k, int metric,
                      const void *ids, const void *dist)
{
    if (!idx) return fail(LPQ_EINVAL, "null index");
    if (nq < 0) return fail(LPQ_EINVAL, "nq < 0");
    if (k < 1) return fail(LPQ_EINVAL, "k = %d < 1", k);
    if (metric != LPQ_METRIC_L2SQ && metric != LPQ_METRIC_IP) return fail(LPQ_EINVAL, "unknown metric %d", metric);
    if (idx->size < 1) return fail(LPQ_ESTATE, "search on an empty index");
    if (k > idx->size) return fail(LPQ_ERANGE, "k = %d > number of items %lld", k, (long long)idx->size);
    if (k > MAX_K) return fail(LPQ_ERANGE, "k = %d > %d", k, (int)MAX_K);
    if (idx->packed && k > MAX_K_PACKED)
        return fail(LPQ_ERANGE, "k = %d > %d, the most a packed index is searched for", k, (int)MAX_K_PACKED);
    if (nq > 0 && (!q || !ids || !dist)) return fail(LPQ_EINVAL, "null argument");
    if (nq > 0 && ld < idx->d) return fail(LPQ_EINVAL, "ld < d");
    if (nq * (int64_t)k >= (int64_t(1) << 40)) return fail(LPQ_ERANGE, "nq too large");
    return LPQ_OK;
}

// Everything after the queries are codes in the workspace.
// qcodes / qnorms: the nq queries' codes (rows of d_pad bytes, zero rows up to a multiple of 512
// readable behind them) and the per-query term of the final distance; emit_mode: how the merge
// turns a key into a distance.
int search_core(const lpq_index *idx, const Plan &p, char *ws, const int8_t *qcodes, const int32_t *qnorms, int64_t nq,
                int k, int metric, int emit_mode, int32_t *ids, int32_t *dist, hipStream_t st)
{
    SearchArgs a;
    a.codes = idx->codes; a.norms = idx->norms; a.cinit = idx->cinit; a.parity = idx->parity;
    a.n = idx->size; a.d_pad = idx->d_pad;
    a.packed = idx->packed;
    a.qcodes = qcodes;
    a.nq = nq; a.k = k; a.metric = metric;
#ifdef LPQ_ABLATION
    a.dry_run = (int)tune(LPQ_TUNE_DRY_RUN);
#endif
    a.work_order = (int)tune(LPQ_TUNE_WORK_ORDER);
    a.wave_queries = 64;
    a.rsplit = p.rsplit;
    a.rs_waves = p.rsplit ? p.rs_waves : 4;
    cand_t *lists1 = reinterpret_cast<cand_t *>(ws + p.off_lists1);
    cand_t *seedlist = reinterpret_cast<cand_t *>(ws + p.off_seedlist);
    cand_t *seeds = reinterpret_cast<cand_t *>(ws + p.off_seeds);
    cand_t *lists2 = reinterpret_cast<cand_t *>(ws + p.off_lists2);
    int32_t *gmax = reinterpret_cast<int32_t *>(ws + p.off_gmax);

    cand_t *merge_tmp = reinterpret_cast<cand_t *>(ws + p.off_merge_tmp);
    // Final merge of the main pass' S2 lists (plus an optional extra list), in one or two passes.
    const bool sorted = p.mode != PLAN_MFMA_LDS;   // that scan's lists come out in arrival order
    auto final_merge = [&](const cand_t *extra) -> hipError_t {
        if (!p.merge_group)
            return launch_merge(lists2, nq, p.S2, k, extra, nullptr, nullptr, ids, dist, qnorms, emit_mode, st, sorted);
        const int groups = (int)ceil_div(p.S2, p.merge_group);
        hipError_t e = launch_merge_groups(lists2, nq, p.S2, p.merge_group, k, merge_tmp, st);
        if (e != hipSuccess) return e;
        return launch_merge(merge_tmp, nq, groups, k, extra, nullptr, nullptr, ids, dist, qnorms, emit_mode, st, true);
    };
    auto scan = [&](int64_t r0, int64_t r1, int S, const cand_t *sd, cand_t *out) -> hipError_t {
        KernelSpan span(st);
        return p.mode == PLAN_GENERIC ? launch_search_generic(a, r0, r1, S, sd, out, st)
                                      : launch_search_mfma(a, r0, r1, S, sd, out, st);
    };
    auto seed_pass = [&]() -> hipError_t {
        {
            KernelSpan span(st, LPQ_PROFILE_SEED);
            a.wave_queries = p.wave_queries;   // same query tiling as the scan it seeds
            hipError_t e = p.piece_stride ? launch_seed_mfma(a, 0, a.n, p.S1, p.SEG, gmax, st, 0, 0, p.piece_stride, p.piece_stages)
                           : p.seed_stride ? launch_seed_mfma(a, 0, a.n, p.S1, p.SEG, gmax, st, p.seed_stride, p.seed_stages)
                                           : launch_seed_mfma(a, 0, p.seed_rows, p.S1, p.SEG, gmax, st);
            a.wave_queries = 64;
            if (e != hipSuccess) return e;
        }
        return launch_seed_finalize(gmax, nq, p.G, k, seeds, st,
                                    p.mode == PLAN_MFMA_COLLECT ? reinterpret_cast<int32_t *>(ws + p.off_qlist) + nq : nullptr);
    };
    if (p.mode == PLAN_MFMA_COLLECT) {
        cand_t *cbuf = reinterpret_cast<cand_t *>(ws + p.off_cbuf);
        int32_t *ccnt = reinterpret_cast<int32_t *>(ws + p.off_ccnt);
        int32_t *over = reinterpret_cast<int32_t *>(ws + p.off_over);
        HIP_TRY(seed_pass());
        {
            KernelSpan span(st);
            a.wave_queries = p.wave_queries;
            hipError_t e = launch_collect_mfma(a, 0, a.n, p.S2, seeds, cbuf, ccnt, p.Cs, st);
            a.wave_queries = 64;
            HIP_TRY(e);
        }
        int32_t *qlist = reinterpret_cast<int32_t *>(ws + p.off_qlist), *qcount = qlist + nq;
        HIP_TRY(launch_collect_select(cbuf, ccnt, nq, p.SS, p.Cs, k, over, qlist, qcount, ids, dist, qnorms, emit_mode, st,
                                      p.expect));
        // Queries whose candidates did not fit are searched again, exactly: a few by the generic kernel;
        // many (a corpus full of duplicates or ties) by a pass of the register-list kernel over the
        // query tiles that hold one.  Both are launched; the count on the device decides which works.
        // (row-split plans - up to 64 queries - never start with the generic kernel: one query there
        // takes longer than a round of the scan for all of them)
        const int few = p.Sr ? REDO_GENERIC_MAX : (p.rounds ? (p.rsplit ? -1 : REFINE_GENERIC_MAX) : INT32_MAX);
        if (few >= 0) {
            HIP_TRY(launch_search_generic_list(a, 0, a.n, p.Sg, qlist, qcount, lists2, st, few));
            HIP_TRY(launch_merge(lists2, nq, p.Sg, k, nullptr, nullptr, nullptr, ids, dist, qnorms, emit_mode, st, false, over,
                                 (p.Sr || p.rounds) ? qcount : nullptr, 0, few));
        }
        if (p.rounds) {
            // Lists too long for the register-list kernel: the flagged queries get bounds from what the
            // scan collected for them and the scan runs again over the query tiles that hold one, up to
            // p.rounds times (what a round collects is the FIRST candidates of each region in scan
            // order, not the best, so one round may still leave too many: each round cuts the number
            // that pass by about k / (candidates the regions hold)).  What overflows even then goes
            // through the generic kernel.  Every launch is gated on the device by the count of queries
            // the round before flagged: more than `few` for the first round, any for the later ones.
            cand_t *bounds2 = reinterpret_cast<cand_t *>(ws + p.off_bounds2);
            const int32_t *over_prev = over, *count_prev = qcount;
            int min_prev = few < 0 ? 0 : few;
            const cand_t *bounds_prev = seeds;
            for (int r = 0; r < p.rounds; ++r) {
                int32_t *over_r = reinterpret_cast<int32_t *>(ws + p.off_over2) + (size_t)r * nq;
                int32_t *qlist_r = reinterpret_cast<int32_t *>(ws + p.off_qlist2) + (size_t)r * (nq + 1), *count_r = qlist_r + nq;
                HIP_TRY(launch_collect_refine(cbuf, ccnt, nq, p.SS, p.Cs, k, over_prev, count_prev, min_prev, bounds_prev,
                                              bounds2, count_r, st));
                SearchArgs ar = a;
                ar.wave_queries = p.wave_queries;
                ar.redo_flags = over_prev; ar.redo_count = count_prev; ar.redo_min = min_prev;
                HIP_TRY(launch_collect_mfma(ar, 0, a.n, p.S2, bounds2, cbuf, ccnt, p.Cs, st));
                HIP_TRY(launch_collect_select(cbuf, ccnt, nq, p.SS, p.Cs, k, over_r, qlist_r, count_r, ids, dist, qnorms,
                                              emit_mode, st, 0, over_prev, count_prev, min_prev));
                over_prev = over_r; count_prev = count_r; min_prev = 0; bounds_prev = bounds2;
                if (r + 1 == p.rounds) {
                    HIP_TRY(launch_search_generic_list(a, 0, a.n, p.Sg, qlist_r, count_r, lists2, st, INT32_MAX));
                    HIP_TRY(launch_merge(lists2, nq, p.Sg, k, nullptr, nullptr, nullptr, ids, dist, qnorms, emit_mode, st,
                                         false, over_r));
                }
            }
        }
        if (p.Sr) {
            cand_t *lists_r = reinterpret_cast<cand_t *>(ws + p.off_redo);
            SearchArgs ar = a;
            ar.rsplit = false;
            ar.wave_queries = 64;
            ar.redo_flags = over; ar.redo_count = qcount; ar.redo_min = REDO_GENERIC_MAX;
            HIP_TRY(launch_search_mfma(ar, 0, a.n, p.Sr, seeds, lists_r, st));
            HIP_TRY(launch_merge(lists_r, nq, p.Sr, k, nullptr, nullptr, nullptr, ids, dist, qnorms, emit_mode, st, false,
                                 over, qcount, REDO_GENERIC_MAX + 1, INT32_MAX));
        }
    } else if (p.mode == PLAN_MFMA_REG) {
        const cand_t *sd = nullptr;
        if (p.seed_rows) {
            HIP_TRY(seed_pass());
            sd = seeds;
        }
        HIP_TRY(scan(0, a.n, p.S2, sd, lists2));
        HIP_TRY(final_merge(nullptr));
    } else if (p.seed_rows) {
        HIP_TRY(scan(0, p.seed_rows, p.S1, nullptr, lists1));
        HIP_TRY(launch_merge(lists1, nq, p.S1, k, nullptr, seedlist, seeds, nullptr, nullptr, nullptr, metric, st, sorted));
        HIP_TRY(scan(p.seed_rows, a.n, p.S2, seeds, lists2));
        HIP_TRY(final_merge(seedlist));
    } else {
        HIP_TRY(scan(0, a.n, p.S2, nullptr, lists2));
        HIP_TRY(final_merge(nullptr));
    }
    return LPQ_OK;
}

// A packed index is searched in tiles of at most 64 queries by the row-split kernel; the workspace
// holds all queries' codes, their permuted copy and per-query terms, then one tile's plan.
struct PackedPlan {
    int64_t nq_pad;
    size_t off_qcodes, off_qnorms, off_qperm, off_qadj, off_tile, total;
};
constexpr int64_t PACKED_TILE = 64;

PackedPlan make_packed_plan(const lpq_index *idx, int64_t nq, int k)
{
    PackedPlan pp;
    const int64_t full = nq < PACKED_TILE ? nq : PACKED_TILE, last = nq % PACKED_TILE;
    const Plan a = make_plan(idx, full, k);
    size_t tile = a.total;
    int64_t tail = a.nq_pad;
    if (last) {
        const Plan b = make_plan(idx, last, k);
        if (b.total > tile) tile = b.total;
        if (b.nq_pad > tail) tail = b.nq_pad;
    }
    pp.nq_pad = ceil_div(nq, PACKED_TILE) * PACKED_TILE + tail;   // every tile may read a whole padded tile
    const Plan whole = make_plan(idx, nq, k);
    if (whole.mode == PLAN_MFMA_COLLECT && !whole.rsplit) {   // large batch: one scan over all queries
        tile = whole.total;
        if (whole.nq_pad > pp.nq_pad) pp.nq_pad = whole.nq_pad;
    }
    size_t o = 0;
    pp.off_qcodes = o; o = align256(o + (size_t)pp.nq_pad * idx->d_pad);
    pp.off_qnorms = o; o = align256(o + (size_t)pp.nq_pad * sizeof(int32_t));
    pp.off_qperm = o;  o = align256(o + (size_t)pp.nq_pad * idx->d_pad);
    pp.off_qadj = o;   o = align256(o + (size_t)pp.nq_pad * sizeof(int32_t));
    pp.off_tile = o;   o = align256(o + tile);
    pp.total = o;
    return pp;
}

int search_packed(const lpq_index *idx, const PackedPlan &pp, char *ws, int64_t nq, int k, int metric, int32_t *ids,
                  int32_t *dist, hipStream_t st)
{
    int8_t *qperm = reinterpret_cast<int8_t *>(ws + pp.off_qperm);
    int32_t *qadj = reinterpret_cast<int32_t *>(ws + pp.off_qadj);
    HIP_TRY(launch_permute_queries(reinterpret_cast<const int8_t *>(ws + pp.off_qcodes), pp.nq_pad, idx->d_pad,
                                   metric == LPQ_METRIC_L2SQ, qperm, qadj, st));
    const int emit = metric == LPQ_METRIC_L2SQ ? MODE_I8_L2 : MODE_I8_IP_ADJ;
    const Plan whole = make_plan(idx, nq, k);
    if (whole.mode == PLAN_MFMA_COLLECT && !whole.rsplit)
        return search_core(idx, whole, ws + pp.off_tile, qperm, qadj, nq, k, metric, emit, ids, dist, st);
    for (int64_t q0 = 0; q0 < nq; q0 += PACKED_TILE) {
        const int64_t nt = nq - q0 < PACKED_TILE ? nq - q0 : PACKED_TILE;
        const Plan pt = make_plan(idx, nt, k);
        int rc = search_core(idx, pt, ws + pp.off_tile, qperm + q0 * idx->d_pad, qadj + q0, nt, k, metric, emit,
                             ids + q0 * k, dist + q0 * k, st);
        if (rc) return rc;
    }
    return LPQ_OK;
}

}  // namespace

extern "C" int lpq_search_plan_info(int d, int bits, int packed, int64_t n_items, int64_t nq, int k, int64_t *out,
                                    int out_count)
{
    if (!out || out_count < LPQ_PLAN_INFO_COUNT) return fail(LPQ_EINVAL, "out must hold LPQ_PLAN_INFO_COUNT values");
    if (d < 1 || bits < 1 || bits > 8) return fail(LPQ_EINVAL, "d < 1 or bits outside 1..8");
    if (d > MAX_D) return fail(LPQ_ERANGE, "d = %d > %d", d, (int)MAX_D);
    if (packed && (bits > 4 || d > MAX_D_PACKED)) return fail(LPQ_EINVAL, "packed storage: at most 4 bits and %d features", (int)MAX_D_PACKED);
    if (n_items < 1 || n_items >= (int64_t(1) << 31) - 1024) return fail(LPQ_ERANGE, "n_items outside 1 .. 2^31 - 1025");
    if (nq < 0 || k < 1) return fail(LPQ_EINVAL, "nq < 0 or k < 1");
    if (k > MAX_K || k > n_items || (packed && k > MAX_K_PACKED)) return fail(LPQ_ERANGE, "k = %d out of range", k);
    lpq_index shape;                     // a description only: no device memory behind it
    shape.d = d; shape.bits = bits; shape.packed = packed != 0;
    shape.d_pad = padded_row_length(d);
    shape.capacity = shape.size = n_items;
    Plan p = make_plan(&shape, nq, k);
    size_t total = p.total, base = 0;
    int64_t nq_rows = p.nq_pad;
    if (shape.packed) {   // searched in tiles of 64 queries unless one collecting scan takes the whole batch
        const PackedPlan pp = make_packed_plan(&shape, nq, k);
        total = pp.total;
        base = pp.off_tile;
        nq_rows = pp.nq_pad;
        if (!(p.mode == PLAN_MFMA_COLLECT && !p.rsplit)) p = make_plan(&shape, nq < PACKED_TILE ? nq : PACKED_TILE, k);
    }
    const int64_t v[LPQ_PLAN_INFO_COUNT] = {
        p.mode, p.rsplit ? 1 : 0, p.rs_waves, p.wave_queries, nq_rows, p.seed_rows, p.S1, p.S2, p.SEG, p.G, p.SS, p.Cs,
        p.Sg, p.Sr, p.rounds, p.merge_group, (int64_t)total, (int64_t)base,
        (int64_t)p.off_qcodes, (int64_t)p.off_qnorms, (int64_t)p.off_lists1, (int64_t)p.off_seedlist, (int64_t)p.off_seeds,
        (int64_t)p.off_lists2, (int64_t)p.off_gmax, (int64_t)p.off_merge_tmp, (int64_t)p.off_cbuf, (int64_t)p.off_ccnt,
        (int64_t)p.off_over, (int64_t)p.off_qlist, (int64_t)p.off_redo, (int64_t)p.off_bounds2, (int64_t)p.off_over2,
        (int64_t)p.off_qlist2, (int64_t)p.total};
    for (int i = 0; i < LPQ_PLAN_INFO_COUNT; ++i) out[i] = v[i];
    return LPQ_OK;
}

extern "C" size_t lpq_search_workspace_bytes(const lpq_index *idx, int64_t nq, int k, int metric)
{
    if (!idx || nq < 0 || k < 1 || k > MAX_K || idx->size < 1 || k > idx->size) return 0;
    (void)metric;
    if (idx->packed) return k > MAX_K_PACKED ? 0 : make_packed_plan(idx, nq, k).total + 256;
    return make_plan(idx, nq, k).total + 256;
}

static int search_f32_queries(const lpq_index *idx, const float *q_dev, int64_t nq, int64_t ld, int k, int metric,
                              int32_t *ids_dev, int32_t *dist_dev, void *workspace_dev, size_t workspace_bytes,
                              hipStream_t st)
{
    char *ws = (char *)workspace_dev;
    if ((uintptr_t)workspace_dev % 256) return fail(LPQ_EINVAL, "workspace must be 256-byte aligned");
    if (idx->packed) {
        const PackedPlan pp = make_packed_plan(idx, nq, k);
        if (!workspace_dev || workspace_bytes < pp.total) return fail(LPQ_ERANGE, "workspace of %zu bytes needed", pp.total);
        HIP_TRY(launch_encode(view(idx->params, idx->d, idx->bits), q_dev, nq, ld,
                              reinterpret_cast<int8_t *>(ws + pp.off_qcodes), idx->d_pad, idx->d_pad,
                              reinterpret_cast<int32_t *>(ws + pp.off_qnorms), st, pp.nq_pad));
        return search_packed(idx, pp, ws, nq, k, metric, ids_dev, dist_dev, st);
    }
    const Plan p = make_plan(idx, nq, k);
    if (!workspace_dev || workspace_bytes < p.total) return fail(LPQ_ERANGE, "workspace of %zu bytes needed", p.total);
    // Padding query rows [nq, nq_pad) are written as zero codes; their results are never written out.
    HIP_TRY(launch_encode(view(idx->params, idx->d, idx->bits), q_dev, nq, ld,
                          reinterpret_cast<int8_t *>(ws + p.off_qcodes), idx->d_pad, idx->d_pad,
                          reinterpret_cast<int32_t *>(ws + p.off_qnorms), st, p.nq_pad));
    return search_core(idx, p, ws, reinterpret_cast<const int8_t *>(ws + p.off_qcodes),
                       reinterpret_cast<const int32_t *>(ws + p.off_qnorms), nq, k, metric, metric, ids_dev, dist_dev, st);
}

extern "C" int lpq_search(const lpq_index *idx, const float *q_dev, int64_t nq, int64_t ld, int k, int metric,
                          int32_t *ids_dev, int32_t *dist_dev, void *workspace_dev, size_t workspace_bytes,
                          void *stream)
{
    int rc = check_search_args(idx, q_dev, nq, ld, k, metric, ids_dev, dist_dev);
    if (rc) return rc;
    if (nq == 0) return LPQ_OK;
    return search_f32_queries(idx, q_dev, nq, ld, k, metric, ids_dev, dist_dev, workspace_dev, workspace_bytes,
                              (hipStream_t)stream);
}

// ---- search without any allocation: the workspace is a device array of the library ----
// One copy of the array exists on every GPU the library is loaded on, at that GPU's own address;
// in host code the array's name is only a handle for hipGetSymbolAddress, never an address.
static __device__ __align__(256) unsigned char scratch[LPQ_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[MAX_DEVICES];   // device address of `scratch` on device i, once looked up

// Device address of `scratch` on the current device (looked up once per device, with that device current).
int scratch_address(void **out)
{
    int dev = -1;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= MAX_DEVICES) return fail(LPQ_EDEVICE, "device ordinal %d outside 0..%d", dev, MAX_DEVICES - 1);
    std::lock_guard<std::mutex> l(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return fail(LPQ_EDEVICE, "hipGetSymbolAddress returned a null address");
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return LPQ_OK;
}
}  // namespace

extern "C" int lpq_search_static(const lpq_index *idx, const float *q_dev, int64_t nq, int64_t ld, int k, int metric,
                                 int32_t *ids_dev, int32_t *dist_dev, void *stream)
{
    int rc = check_search_args(idx, q_dev, nq, ld, k, metric, ids_dev, dist_dev);
    if (rc) return rc;
    if (nq == 0) return LPQ_OK;
    const size_t need = idx->packed ? make_packed_plan(idx, nq, k).total : make_plan(idx, nq, k).total;
    if (need > (size_t)LPQ_STATIC_WORKSPACE_BYTES)
        return fail(LPQ_ERANGE, "this search needs %zu bytes of workspace, the built-in one holds %zu: use lpq_search",
                    need, (size_t)LPQ_STATIC_WORKSPACE_BYTES);
    void *ws = nullptr;
    rc = scratch_address(&ws);
    if (rc) return rc;
    return search_f32_queries(idx, q_dev, nq, ld, k, metric, ids_dev, dist_dev, ws, (size_t)LPQ_STATIC_WORKSPACE_BYTES,
                              (hipStream_t)stream);
}

extern "C" int lpq_search_overflow_stats(const lpq_index *idx, int64_t nq, int k, int metric, const void *workspace_dev,
                                         int64_t *redone_queries, int64_t *max_region_fill)
{
    (void)metric;
    if (!idx || !workspace_dev || !redone_queries || !max_region_fill || nq < 1 || k < 1) return fail(LPQ_EINVAL, "bad argument");
    *redone_queries = 0;
    *max_region_fill = 0;
    const Plan p = make_plan(idx, nq, k);
    if (p.mode != PLAN_MFMA_COLLECT) return LPQ_OK;
    HIP_TRY(hipDeviceSynchronize());
    std::vector<int32_t> over((size_t)nq), cnt((size_t)nq * p.SS);
    const char *ws = static_cast<const char *>(workspace_dev) + (idx->packed ? make_packed_plan(idx, nq, k).off_tile : 0);
    HIP_TRY(hipMemcpy(over.data(), ws + p.off_over, over.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
    HIP_TRY(hipMemcpy(cnt.data(), ws + p.off_ccnt, cnt.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
    for (int32_t v : over) *redone_queries += v != 0;
    for (int32_t v : cnt) if (v > *max_region_fill) *max_region_fill = v;
    return LPQ_OK;
}

extern "C" int lpq_search_overflow_left(const lpq_index *idx, int64_t nq, int k, int metric, const void *workspace_dev,
                                        int64_t *left_queries)
{
    (void)metric;
    if (!idx || !workspace_dev || !left_queries || nq < 1 || k < 1) return fail(LPQ_EINVAL, "bad argument");
    *left_queries = 0;
    const Plan p = make_plan(idx, nq, k);
    if (p.mode != PLAN_MFMA_COLLECT || !p.rounds) return LPQ_OK;
    HIP_TRY(hipDeviceSynchronize());
    std::vector<int32_t> over2((size_t)nq);
    const char *ws = static_cast<const char *>(workspace_dev) + (idx->packed ? make_packed_plan(idx, nq, k).off_tile : 0);
    HIP_TRY(hipMemcpy(over2.data(), ws + p.off_over2 + (size_t)(p.rounds - 1) * nq * sizeof(int32_t),
                      over2.size() * sizeof(int32_t), hipMemcpyDeviceToHost));
    for (int32_t v : over2) *left_queries += v != 0;
    return LPQ_OK;
}

extern "C" int lpq_search_i8(const lpq_index *idx, const int8_t *qcodes_dev, int64_t nq, int64_t ld, int k,
                             int metric, int32_t *ids_dev, int32_t *dist_dev, void *workspace_dev,
                             size_t workspace_bytes, void *stream)
{
    int rc = check_search_args(idx, qcodes_dev, nq, ld, k, metric, ids_dev, dist_dev);
    if (rc) return rc;
    if (nq == 0) return LPQ_OK;
    hipStream_t st = (hipStream_t)stream;
    char *ws = (char *)workspace_dev;
    if ((uintptr_t)workspace_dev % 256) return fail(LPQ_EINVAL, "workspace must be 256-byte aligned");
    if (idx->packed) {
        const PackedPlan pp = make_packed_plan(idx, nq, k);
        if (!workspace_dev || workspace_bytes < pp.total) return fail(LPQ_ERANGE, "workspace of %zu bytes needed", pp.total);
        HIP_TRY(launch_repack_i8(qcodes_dev, nq, ld, idx->d, reinterpret_cast<int8_t *>(ws + pp.off_qcodes), idx->d_pad,
                                 idx->d_pad, reinterpret_cast<int32_t *>(ws + pp.off_qnorms), st, pp.nq_pad));
        return search_packed(idx, pp, ws, nq, k, metric, ids_dev, dist_dev, st);
    }
    const Plan p = make_plan(idx, nq, k);
    if (!workspace_dev || workspace_bytes < p.total) return fail(LPQ_ERANGE, "workspace of %zu bytes needed", p.total);
    HIP_TRY(launch_repack_i8(qcodes_dev, nq, ld, idx->d, reinterpret_cast<int8_t *>(ws + p.off_qcodes), idx->d_pad,
                             idx->d_pad, reinterpret_cast<int32_t *>(ws + p.off_qnorms), st, p.nq_pad));
    return search_core(idx, p, ws, reinterpret_cast<const int8_t *>(ws + p.off_qcodes),
                       reinterpret_cast<const int32_t *>(ws + p.off_qnorms), nq, k, metric, metric, ids_dev, dist_dev, st);
}

// -------------------------------------------------------------------- fp32 exact ----
extern "C" size_t lpq_search_f32_workspace_bytes(int64_t n, int64_t nq, int d, int k)
{
    if (n < 1 || nq < 0 || d < 1 || k < 1 || k > MAX_K || k > n || d > f32_max_d(k)) return 0;
    return f32_workspace_bytes(n, nq, d, k) + 256;
}

extern "C" int lpq_search_f32(const float *x_dev, int64_t n, int64_t ldx, const float *q_dev, int64_t nq,
                              int64_t ldq, int d, int k, int metric, int32_t *ids_dev, float *dist_dev,
                              void *workspace_dev, size_t workspace_bytes, void *stream)
{
    if (d < 1) return fail(LPQ_EINVAL, "d < 1");
    if (n < 1) return fail(LPQ_ESTATE, "no items");
    if (nq < 0) return fail(LPQ_EINVAL, "nq < 0");
    if (k < 1) return fail(LPQ_EINVAL, "k < 1");
    if (metric != LPQ_METRIC_L2SQ && metric != LPQ_METRIC_IP) return fail(LPQ_EINVAL, "unknown metric %d", metric);
    if (k > n || k > MAX_K) return fail(LPQ_ERANGE, "k = %d out of range", k);
    if (n >= (int64_t(1) << 31) - 1024) return fail(LPQ_ERANGE, "n must stay below 2^31 - 1024");
    if (d > f32_max_d(k))
        return fail(LPQ_ERANGE, "d = %d: the fp32 search takes at most %d features for k = %d", d, f32_max_d(k), k);
    if (nq == 0) return LPQ_OK;
    if (!x_dev || !q_dev || !ids_dev || !dist_dev) return fail(LPQ_EINVAL, "null argument");
    if (ldx < d || ldq < d) return fail(LPQ_EINVAL, "row stride smaller than d");
    const size_t need = f32_workspace_bytes(n, nq, d, k);
    if (!workspace_dev || workspace_bytes < need) return fail(LPQ_ERANGE, "workspace of %zu bytes needed", need);
    if ((uintptr_t)workspace_dev % 256) return fail(LPQ_EINVAL, "workspace must be 256-byte aligned");
    HIP_TRY(launch_search_f32(x_dev, n, ldx, q_dev, nq, ldq, d, k, metric, ids_dev, dist_dev, workspace_dev,
                              (hipStream_t)stream));
    return LPQ_OK;
}
