// Attainable-rate probes for benchmarks: what this GPU sustains on the two resources that bound
// the search (the int8 matrix pipe and the stream of corpus bytes into a CU), measured with
// kernels that do nothing else.  They put the roofline fractions of the scan kernels, which are
// quoted against the published peaks, next to what the part reaches in practice: the matrix
// rate depends on the operand bits (the shader clock falls under matrix load, more so when many
// operand bits toggle), the streaming rate on the path the bytes take into the CU.
#include "mfma_common.h"

namespace lpq {

namespace {

// Register-resident loop of v_mfma_i32_32x32x32_i8: two chains of four instructions per
// iteration, operands loaded once from `data` (n16 16-byte words, wrapped), no memory traffic
// inside the loop.  Four waves per workgroup, two workgroups per CU, as the scan kernels run.
__global__ __launch_bounds__(256, 2) void probe_mfma_kernel(const v4i *__restrict__ data, size_t n16,
                                                             int *__restrict__ sink, int iters)
{
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    v4i A[4], B[2][4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        A[i] = data ? data[(t * 12 + i) % n16] : v4i{0, 0, 0, 0};
        B[0][i] = data ? data[(t * 12 + 4 + i) % n16] : v4i{0, 0, 0, 0};
        B[1][i] = data ? data[(t * 12 + 8 + i) % n16] : v4i{0, 0, 0, 0};
    }
    v16i c0;
#pragma unroll
    for (int i = 0; i < 16; ++i) c0[i] = 0;
    int res = 0;
    for (int it = 0; it < iters; ++it) {
        v16i acc[2];
#pragma unroll
        for (int ks = 0; ks < 4; ++ks)
#pragma unroll
            for (int nb = 0; nb < 2; ++nb)
                acc[nb] = __builtin_amdgcn_mfma_i32_32x32x32_i8(A[ks], B[nb][ks], ks == 0 ? c0 : acc[nb], 0, 0, 0);
        res += acc[0][0] + acc[1][5];
        A[0][0] ^= (res & 1);   // keeps the loop from being hoisted; flips one operand bit at most
    }
    sink[t] = res;
}

// Streaming read of `chunks` blocks of 4 KB through the asynchronous global->LDS path the scan
// kernels use: every wave has a private ring of RING slots of 4 KB, copies chunk c + RING - 1
// while it waits for chunk c (counted s_waitcnt vmcnt, no workgroup barrier), and reads 16 bytes
// per lane of each landed chunk from LDS.  Workgroup w, wave v take chunks (4 w + v), + 4 * grid, ...
constexpr int PROBE_RING = 3;
__global__ __launch_bounds__(256, 2) void probe_stream_lds_kernel(const unsigned char *__restrict__ src, int64_t chunks,
                                                                   int *__restrict__ sink)
{
    __shared__ __align__(16) unsigned char ring[4][PROBE_RING][4096];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t first = (int64_t)blockIdx.x * 4 + wave, step = (int64_t)gridDim.x * 4;
    const int64_t mine = first < chunks ? (chunks - first + step - 1) / step : 0;   // chunks this wave takes
    const unsigned base = lds_offset(&ring[wave][0][0]);
    __builtin_amdgcn_s_waitcnt(0x0F70);   // only the copies below count from here on
    auto issue = [&](int64_t i) {
        const unsigned char *g = src + (first + i * step) * 4096 + lane * 16;
        const unsigned slot = base + (unsigned)(i % PROBE_RING) * 4096;
#pragma unroll
        for (int j = 0; j < 4; ++j) async_copy16(g + j * 1024, slot + j * 1024);
    };
    for (int64_t i = 0; i < PROBE_RING - 1 && i < mine; ++i) issue(i);
    int acc = 0;
    for (int64_t i = 0; i < mine; ++i) {
        const int64_t last = mine - 1 < i + PROBE_RING - 2 ? mine - 1 : i + PROBE_RING - 2;   // newest chunk issued so far
        wait_vmcnt((int)(last - i) * 4);                                     // chunk i has landed
        const v4i v = *reinterpret_cast<const v4i *>(&ring[wave][i % PROBE_RING][lane * 16]);
        acc ^= v[0] ^ v[1] ^ v[2] ^ v[3];
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");                   // read done before the slot is refilled
        if (i + PROBE_RING - 1 < mine) issue(i + PROBE_RING - 1);            // into the slot chunk i - 1 was read from
    }
    sink[(size_t)blockIdx.x * 256 + threadIdx.x] = acc;
}

// The same bytes through ordinary 16-byte register loads, grid-stride.
__global__ __launch_bounds__(256) void probe_stream_reg_kernel(const v4i *__restrict__ src, int64_t n16, int *__restrict__ sink)
{
    const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x, step = (int64_t)gridDim.x * 256;
    int acc = 0;
    int64_t i = t;
    for (; i + 3 * step < n16; i += 4 * step) {
        const v4i a = src[i], b = src[i + step], c = src[i + 2 * step], d = src[i + 3 * step];
        acc ^= a[0] ^ a[1] ^ a[2] ^ a[3] ^ b[0] ^ b[1] ^ b[2] ^ b[3] ^ c[0] ^ c[1] ^ c[2] ^ c[3] ^ d[0] ^ d[1] ^ d[2] ^ d[3];
    }
    for (; i < n16; i += step) {
        const v4i a = src[i];
        acc ^= a[0] ^ a[1] ^ a[2] ^ a[3];
    }
    sink[t] = acc;
}

// The inner loop of the wide collecting scan with nothing around it: per 32-row block four chains of
// four matrix instructions (128 queries per wave, query operands in registers), the filter epilogue of
// a chain (max tree, compare, branch) one chain later, row operands and accumulator seeds read from a
// two-stage LDS ring that is filled once, before the loop - no copies, no barrier, no candidates (the
// threshold is never reached).  What this sustains is the ceiling of the scan's loop on this GPU for
// operand bits like those in `data`; the scan itself adds the corpus copies, a barrier per stage, the
// candidate path and the padding of the query batch.
__global__ __launch_bounds__(256, 2) void probe_scan_core_kernel(const v4i *__restrict__ data, size_t n16,
                                                                  int *__restrict__ sink, int stages)
{
    extern __shared__ __align__(16) unsigned char smem[];   // ring 2 x 128 rows x 128 B, accumulator seeds 2 x 132 ints, a dump area
    constexpr int RING = 32768, AUX = 1056;
    const int lane = threadIdx.x & 63, col = lane & 31, half = lane >> 5;
    const size_t t = (size_t)blockIdx.x * 256 + threadIdx.x;
    for (int i = threadIdx.x; i < RING / 16; i += 256)
        reinterpret_cast<v4i *>(smem)[i] = data ? data[(size_t)i % n16] : v4i{0, 0, 0, 0};
    for (int i = threadIdx.x; i < AUX / 4; i += 256) reinterpret_cast<int *>(smem + RING)[i] = -(i * 37 & 0xFFFF);
    __syncthreads();
    v4i B[4][4];
#pragma unroll
    for (int nb = 0; nb < 4; ++nb)
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) B[nb][ks] = data ? data[(t * 16 + nb * 4 + ks) % n16] : v4i{0, 0, 0, 0};
    int a_off[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) a_off[ks] = col * 128 + (((2 * ks + half) ^ (col & 7)) * 16);
    const int thr = INT32_MAX;
    int qcnt = 0;
    const int *aux = reinterpret_cast<const int *>(smem + RING);
    v4i A0[4], A1[4];
    v16i C0 = {}, C1 = {};
    unsigned P0 = 0, P1 = 0;
    v16i carry = {};
    bool have_carry = false;
#define PROBE_LOAD(TT, BLK, AREG, CREG, PREG)                                                           \
    do {                                                                                                \
        const unsigned char *sb_ = smem + ((TT) & 1) * 16384 + (BLK) * 4096;                            \
        const int *cb_ = aux + ((TT) & 1) * 132;                                                        \
        _Pragma("unroll") for (int ks = 0; ks < 4; ++ks) AREG[ks] = *reinterpret_cast<const v4i *>(sb_ + a_off[ks]); \
        _Pragma("unroll") for (int g = 0; g < 4; ++g) {                                                 \
            const v4i v_ = *reinterpret_cast<const v4i *>(cb_ + (BLK) * 32 + 8 * g + 4 * half);         \
            CREG[4 * g] = v_[0]; CREG[4 * g + 1] = v_[1]; CREG[4 * g + 2] = v_[2]; CREG[4 * g + 3] = v_[3]; \
        }                                                                                               \
        PREG = (unsigned)cb_[128 + (BLK)];                                                              \
    } while (0)
#define PROBE_EPI(VEC)                                                                                  \
    do {                                                                                                \
        const v16i v = (VEC);                                                                           \
        int m = max(max(v[0], v[1]), v[2]);                                                             \
        m = max(max(m, v[3]), v[4]); m = max(max(m, v[5]), v[6]); m = max(max(m, v[7]), v[8]);          \
        m = max(max(m, v[9]), v[10]); m = max(max(m, v[11]), v[12]); m = max(max(m, v[13]), v[14]);     \
        m = max(m, v[15]);                                                                              \
        const bool trip = m >= thr;                                                                     \
        const unsigned long long mask = __ballot(trip);                                                 \
        __builtin_amdgcn_sched_group_barrier(0x008, 2, 0);                                              \
        __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);                                              \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                              \
        __builtin_amdgcn_sched_group_barrier(0x002, 5, 0);                                              \
        __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);                                              \
        if (__builtin_expect(mask != 0, 0)) {   /* never taken: the candidate path, kept as code */     \
            const int below = __builtin_amdgcn_mbcnt_hi((unsigned)(mask >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)mask, 0u)); \
            if (trip) {                                                                                 \
                v4i *dst_ = reinterpret_cast<v4i *>(smem + RING + AUX + 32 + ((qcnt + below) & 63) * 64); \
                _Pragma("unroll") for (int g = 0; g < 4; ++g) dst_[g] = v4i{v[4 * g], v[4 * g + 1], v[4 * g + 2], v[4 * g + 3]}; \
            }                                                                                           \
            qcnt += __popcll(mask);                                                                     \
        }                                                                                               \
    } while (0)
#define PROBE_CHAIN(NBI, AREG, CREG)                                                                    \
    _Pragma("unroll") for (int ks = 0; ks < 4; ++ks)                                                    \
        acc[NBI] = __builtin_amdgcn_mfma_i32_32x32x32_i8(AREG[ks], B[NBI][ks], ks == 0 ? CREG : acc[NBI], 0, 0, 0)
#define PROBE_BLOCK(AREG, CREG)                                                                         \
    do {                                                                                                \
        v16i acc[4];                                                                                    \
        PROBE_CHAIN(0, AREG, CREG);                                                                     \
        if (have_carry) PROBE_EPI(carry);                                                               \
        PROBE_CHAIN(1, AREG, CREG); PROBE_EPI(acc[0]);                                                  \
        PROBE_CHAIN(2, AREG, CREG); PROBE_EPI(acc[1]);                                                  \
        PROBE_CHAIN(3, AREG, CREG); PROBE_EPI(acc[2]);                                                  \
        carry = acc[3]; have_carry = true;                                                              \
    } while (0)
    PROBE_LOAD(0, 0, A0, C0, P0);
    for (int st = 0; st < stages; ++st) {
        PROBE_LOAD(st, 1, A1, C1, P1); PROBE_BLOCK(A0, C0);
        PROBE_LOAD(st, 2, A0, C0, P0); PROBE_BLOCK(A1, C1);
        PROBE_LOAD(st, 3, A1, C1, P1); PROBE_BLOCK(A0, C0);
        PROBE_LOAD(st + 1, 0, A0, C0, P0); PROBE_BLOCK(A1, C1);
    }
    if (have_carry) PROBE_EPI(carry);
#undef PROBE_LOAD
#undef PROBE_EPI
#undef PROBE_CHAIN
#undef PROBE_BLOCK
    sink[t] = qcnt + (int)(P0 + P1);
}

struct Timer {
    hipEvent_t a = nullptr, b = nullptr;
    ~Timer()
    {
        if (a) (void)hipEventDestroy(a);
        if (b) (void)hipEventDestroy(b);
    }
};

}  // namespace

hipError_t probe_mfma(const void *operands, size_t bytes, int iters, double *tops, hipStream_t st)
{
    constexpr int BLOCKS = 1024;
    int *sink = nullptr;
    hipError_t e = hipMalloc(&sink, (size_t)BLOCKS * 256 * sizeof(int));
    if (e != hipSuccess) return e;
    Timer t;
    e = hipEventCreate(&t.a);
    if (e == hipSuccess) e = hipEventCreate(&t.b);
    if (e == hipSuccess) {
        const v4i *data = reinterpret_cast<const v4i *>(operands);
        const size_t n16 = bytes / 16;
        probe_mfma_kernel<<<BLOCKS, 256, 0, st>>>(data, n16, sink, iters / 8 + 1);   // warm-up
        e = hipEventRecord(t.a, st);
        probe_mfma_kernel<<<BLOCKS, 256, 0, st>>>(data, n16, sink, iters);
        if (e == hipSuccess) e = hipEventRecord(t.b, st);
        if (e == hipSuccess) e = hipEventSynchronize(t.b);
        if (e == hipSuccess) e = hipGetLastError();
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, t.a, t.b);
        if (e == hipSuccess) *tops = (double)BLOCKS * 4 * iters * 8 * 65536.0 / (ms * 1e-3) / 1e12;
    }
    (void)hipFree(sink);
    return e;
}

hipError_t probe_scan_core(const void *operands, size_t bytes, int stages, double *tops, hipStream_t st)
{
    constexpr int BLOCKS = 512;                  // two workgroups per CU, all resident
    constexpr size_t LDS = 70 * 1024;            // the scan's footprint, which is what holds a CU to two workgroups
    int *sink = nullptr;
    hipError_t e = hipMalloc(&sink, (size_t)BLOCKS * 256 * sizeof(int));
    if (e != hipSuccess) return e;
    Timer t;
    e = hipEventCreate(&t.a);
    if (e == hipSuccess) e = hipEventCreate(&t.b);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(probe_scan_core_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess) {
        const v4i *data = reinterpret_cast<const v4i *>(operands);
        const size_t n16 = bytes / 16;
        probe_scan_core_kernel<<<BLOCKS, 256, LDS, st>>>(data, n16, sink, stages / 8 + 1);   // warm-up
        e = hipEventRecord(t.a, st);
        probe_scan_core_kernel<<<BLOCKS, 256, LDS, st>>>(data, n16, sink, stages);
        if (e == hipSuccess) e = hipEventRecord(t.b, st);
        if (e == hipSuccess) e = hipEventSynchronize(t.b);
        if (e == hipSuccess) e = hipGetLastError();
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, t.a, t.b);
        if (e == hipSuccess) *tops = (double)BLOCKS * 4 * stages * 64 * 65536.0 / (ms * 1e-3) / 1e12;
    }
    (void)hipFree(sink);
    return e;
}

hipError_t probe_stream(const void *src, size_t bytes, int mode, int reps, double *gbps, hipStream_t st)
{
    constexpr int BLOCKS = 512;
    int *sink = nullptr;
    hipError_t e = hipMalloc(&sink, (size_t)BLOCKS * 4 * 256 * sizeof(int));
    if (e != hipSuccess) return e;
    Timer t;
    e = hipEventCreate(&t.a);
    if (e == hipSuccess) e = hipEventCreate(&t.b);
    if (e == hipSuccess) {
        for (int r = 0; r <= reps && e == hipSuccess; ++r) {   // first pass untimed
            if (r == 1) e = hipEventRecord(t.a, st);
            if (mode == 0)
                probe_stream_lds_kernel<<<BLOCKS, 256, 0, st>>>(static_cast<const unsigned char *>(src), (int64_t)(bytes / 4096), sink);
            else
                probe_stream_reg_kernel<<<BLOCKS * 4, 256, 0, st>>>(static_cast<const v4i *>(src), (int64_t)(bytes / 16), sink);
        }
        if (e == hipSuccess) e = hipEventRecord(t.b, st);
        if (e == hipSuccess) e = hipEventSynchronize(t.b);
        if (e == hipSuccess) e = hipGetLastError();
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, t.a, t.b);
        if (e == hipSuccess) *gbps = (double)bytes * reps / (ms * 1e-3) / 1e9;
    }
    (void)hipFree(sink);
    return e;
}

}  // namespace lpq
