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
