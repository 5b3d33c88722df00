// Host-side checks meant to run under AddressSanitizer + UndefinedBehaviorSanitizer, without a GPU:
//   1. the CPU oracle's C functions on small inputs, with the edge cases of the method (one item,
//      k = n, NaN / infinities, constant features, absent ids);
//   2. the planner of liblpq.so through lpq_search_plan_info over a grid of shapes: every call
//      returns, no integer trap, every buffer offset is 256-byte aligned, used offsets never
//      decrease and end inside the total;
//   3. argument checks of the C ABI that come before any device work.
// usage: san_driver <path to the sanitized liblpq>      exit status 0 = all checks passed
#include <dlfcn.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <cmath>
#include <vector>

#include "lpq.h"   // declarations only: the library itself is loaded with dlopen

extern "C" {
void lpqo_derive_m(const float *sb, const float *se, int d, int bits, float *m);
int lpqo_calibrate(const float *x, int64_t n, int64_t ld, int d, int bits, int mode, int scope, double sigma_mult,
                   float *k, float *sb, float *se, float *m);
void lpqo_encode(const float *x, int64_t n, int64_t ld, int d, int bits, const float *k, const float *sb,
                 const float *se, const float *m, int8_t *codes, int64_t ldc, int32_t *norms);
int32_t lpqo_dist_l2sq(const int8_t *a, const int8_t *b, int d);
int32_t lpqo_dist_ip(const int8_t *a, const int8_t *b, int d);
int lpqo_search_i8(const int8_t *codes, int64_t n, int64_t ldc, const int8_t *q, int64_t nq, int64_t ldq, int d, int k,
                   int metric, int32_t *ids, int32_t *dists, int threads);
int lpqo_search_f32(const float *x, int64_t n, int64_t ldx, const float *q, int64_t nq, int64_t ldq, int d, int k,
                    int metric, int32_t *ids, float *dists, int threads);
void lpqo_gather_dist(const int8_t *codes, int64_t ldc, const int8_t *q, int64_t nq, int64_t ldq, int d,
                      const int32_t *ids, int m, int metric, int32_t *out);
int lpqo_rerank_f32(const float *x, int64_t ldx, const float *q, int64_t nq, int64_t ldq, int d, const int32_t *cand,
                    int kc, int k, int metric, int32_t *ids, float *dists);
double lpqo_recall(const int32_t *approx, const int32_t *exact, int64_t nq, int k);
}

static int g_fail = 0;
#define CHECK(cond, ...)                                                            \
    do {                                                                            \
        if (!(cond)) {                                                              \
            if (++g_fail <= 20) { printf("FAIL %s:%d: ", __FILE__, __LINE__); printf(__VA_ARGS__); printf("\n"); } \
        }                                                                           \
    } while (0)

static uint64_t g_rng = 0x9E3779B97F4A7C15ull;
static double unif() { g_rng = g_rng * 6364136223846793005ull + 1442695040888963407ull; return (double)(g_rng >> 11) / 9007199254740992.0; }

static void oracle_checks()
{
    const int ns[] = {1, 7, 64}, ds[] = {1, 5, 33}, bitss[] = {1, 3, 8};
    for (int n : ns) for (int d : ds) for (int bits : bitss) for (int mode = 0; mode < 4; ++mode) for (int scope = 0; scope < 3; ++scope) {
        const int ld = d + 2, nq = 3;
        std::vector<float> x((size_t)n * ld), q((size_t)nq * ld), k(d), sb(d), se(d), m(d);
        for (auto &v : x) v = (float)(unif() * 2.0 - 1.0);
        for (auto &v : q) v = (float)(unif() * 2.0 - 1.0);
        if (d > 1) for (int i = 0; i < n; ++i) x[(size_t)i * ld + 1] = 0.25f;            // a constant feature
        const double arg = mode == 3 ? 0.1 : 1.0;
        int rc = lpqo_calibrate(x.data(), n, ld, d, bits, mode, scope, arg, k.data(), sb.data(), se.data(), m.data());
        CHECK(rc == 0, "calibrate rc %d (n %d d %d bits %d mode %d scope %d)", rc, n, d, bits, mode, scope);
        q[0] = NAN; q[1 % (nq * ld)] = INFINITY; q[ld] = -INFINITY;                     // encode maps these, calibrate never sees them
        std::vector<int8_t> cx((size_t)n * d), cq((size_t)nq * d);
        std::vector<int32_t> nx(n), nqn(nq);
        lpqo_encode(x.data(), n, ld, d, bits, k.data(), sb.data(), se.data(), m.data(), cx.data(), d, nx.data());
        lpqo_encode(q.data(), nq, ld, d, bits, k.data(), sb.data(), se.data(), m.data(), cq.data(), d, nqn.data());
        for (int i = 0; i < n; ++i) {
            int64_t s = 0;
            for (int j = 0; j < d; ++j) s += (int64_t)cx[(size_t)i * d + j] * cx[(size_t)i * d + j];
            CHECK(s == nx[i], "norm of row %d", i);
        }
        for (int metric = 0; metric < 2; ++metric) for (int kk : {1, n}) {
            std::vector<int32_t> ids((size_t)nq * kk), dist((size_t)nq * kk);
            rc = lpqo_search_i8(cx.data(), n, d, cq.data(), nq, d, d, kk, metric, ids.data(), dist.data(), 1);
            CHECK(rc == 0, "search_i8 rc %d", rc);
            for (int i = 0; i < nq; ++i) for (int r = 0; r < kk; ++r) {
                const int32_t id = ids[(size_t)i * kk + r];
                CHECK(id >= 0 && id < n, "id out of range");
                if (id < 0 || id >= n) continue;
                const int32_t want = metric == 0 ? lpqo_dist_l2sq(cq.data() + (size_t)i * d, cx.data() + (size_t)id * d, d)
                                                 : lpqo_dist_ip(cq.data() + (size_t)i * d, cx.data() + (size_t)id * d, d);
                CHECK(want == dist[(size_t)i * kk + r], "reported distance is the pair's distance");
                if (r > 0) {
                    const int32_t a = dist[(size_t)i * kk + r - 1], b = dist[(size_t)i * kk + r];
                    CHECK(metric == 0 ? a <= b : a >= b, "rows sorted best first");
                }
            }
            std::vector<int32_t> gid((size_t)nq * 4), gout((size_t)nq * 4);
            for (size_t i = 0; i < gid.size(); ++i) gid[i] = (i % 4 == 3) ? -1 : (int32_t)(unif() * n) % n;
            lpqo_gather_dist(cx.data(), d, cq.data(), nq, d, d, gid.data(), 4, metric, gout.data());
            std::vector<float> fd((size_t)nq * kk);
            std::vector<int32_t> fid((size_t)nq * kk);
            std::vector<float> qf(q);
            for (auto &v : qf) if (!std::isfinite(v)) v = 0.5f;
            rc = lpqo_search_f32(x.data(), n, ld, qf.data(), nq, ld, d, kk, metric, fid.data(), fd.data(), 1);
            CHECK(rc == 0, "search_f32 rc %d", rc);
            std::vector<int32_t> rid((size_t)nq * kk);
            std::vector<float> rd((size_t)nq * kk);
            rc = lpqo_rerank_f32(x.data(), ld, qf.data(), nq, ld, d, ids.data(), kk, kk, metric, rid.data(), rd.data());
            CHECK(rc == 0, "rerank rc %d", rc);
            const double rec = lpqo_recall(ids.data(), fid.data(), nq, kk);
            CHECK(rec >= 0.0 && rec <= 1.0, "recall in [0, 1]");
            if (kk == n) CHECK(rec == 1.0, "k = n: both sets are the whole corpus");
        }
    }
    printf("oracle: calibrate / encode / search / gather / rerank / recall exercised\n");
}

typedef decltype(&lpq_search_plan_info) plan_info_fn;
static const int PLAN_N = LPQ_PLAN_INFO_COUNT;

static void planner_checks(void *lib)
{
    plan_info_fn plan = (plan_info_fn)dlsym(lib, "lpq_search_plan_info");
    CHECK(plan != nullptr, "lpq_search_plan_info not exported");
    if (!plan) return;
    const int ds[] = {1, 31, 32, 64, 65, 96, 100, 128, 129, 160, 192, 224, 256, 257, 384, 500, 512, 768, 1000, 1024, 1025, 1536, 1537, 32768};
    const int bitss[] = {1, 2, 4, 8};
    const int64_t ns[] = {1, 2, 63, 64, 511, 512, 1000, 4095, 4096, 10000, 65535, 65536, 262143, 1000000, 10000000,
                          100000000, (int64_t(1) << 31) - 1025};
    const int64_t nqs[] = {0, 1, 2, 16, 63, 64, 65, 128, 129, 255, 256, 257, 511, 512, 513, 1000, 1025, 2000, 4097, 10000, 200000, 3000000};
    const int ks[] = {1, 2, 3, 10, 11, 16, 17, 24, 25, 32, 33, 100, 128, 129, 500, 1024};
    long calls = 0;
    for (int d : ds) for (int bits : bitss) for (int packed = 0; packed < 2; ++packed) {
        if (packed && (bits > 4 || d > 256)) continue;
        for (int64_t n : ns) for (int64_t nq : nqs) for (int k : ks) {
            if (k > n || (packed && k > 128)) continue;
            int64_t v[PLAN_N];
            for (auto &e : v) e = -12345;
            const int rc = plan(d, bits, packed, n, nq, k, v, PLAN_N);
            ++calls;
            CHECK(rc == 0, "plan rc %d for d %d bits %d packed %d n %lld nq %lld k %d", rc, d, bits, packed, (long long)n, (long long)nq, k);
            if (rc) continue;
#define SHAPE "(d %d bits %d packed %d n %lld nq %lld k %d)", d, bits, packed, (long long)n, (long long)nq, k
            CHECK(v[0] >= 0 && v[0] <= 3, "mode " SHAPE);
            CHECK(v[3] == 32 || v[3] == 64 || v[3] == 128, "queries per wave " SHAPE);
            if (v[3] == 32) CHECK(d > 512 && d <= 1536 && v[0] == 3 && !packed, "32 queries per wave: rows of 768, 1024 or 1536 bytes only " SHAPE);
            CHECK(v[4] >= nq && v[4] >= 1, "query rows cover the batch " SHAPE);
            CHECK(v[5] >= 0 && v[5] <= n, "seeding rows within the corpus " SHAPE);
            CHECK(v[7] >= 1, "at least one split " SHAPE);
            if (v[5] > 0) CHECK(v[6] >= 1, "seeding pass has splits " SHAPE);
            if (v[0] == 3) CHECK(v[10] >= 1 && v[11] >= 1 && v[5] > 0, "collecting scan has regions and a seeding pass " SHAPE);
            CHECK(v[16] > 0 && v[16] < (int64_t(1) << 46), "workspace size sane " SHAPE);
            CHECK(v[17] % 256 == 0 && v[17] + v[34] <= v[16], "tile plan inside the workspace " SHAPE);
            int64_t prev = 0;
            for (int i = 18; i <= 34; ++i) {
                CHECK(v[i] % 256 == 0, "offset %d aligned " SHAPE, i);
                if (v[i] == 0 && i != 18 && i != 34) continue;      // not used by this plan
                CHECK(v[i] >= prev, "offset %d does not decrease " SHAPE, i);
                CHECK(v[i] <= v[34], "offset %d inside the plan " SHAPE, i);
                prev = v[i];
            }
#undef SHAPE
        }
    }
    // argument checks
    int64_t v[PLAN_N];
    CHECK(plan(0, 8, 0, 10, 1, 1, v, PLAN_N) != 0, "d = 0 rejected");
    CHECK(plan(8, 9, 0, 10, 1, 1, v, PLAN_N) != 0, "bits = 9 rejected");
    CHECK(plan(8, 8, 1, 10, 1, 1, v, PLAN_N) != 0, "packed with 8 bits rejected");
    CHECK(plan(8, 8, 0, 10, 1, 11, v, PLAN_N) != 0, "k > n rejected");
    CHECK(plan(8, 8, 0, 10, -1, 1, v, PLAN_N) != 0, "nq < 0 rejected");
    CHECK(plan(8, 8, 0, 10, 1, 1, v, 3) != 0, "short output rejected");
    CHECK(plan(8, 8, 0, 10, 1, 1, nullptr, PLAN_N) != 0, "null output rejected");
    printf("planner: %ld plans checked\n", calls);
}

static void abi_checks(void *lib)
{
    typedef decltype(&lpq_quantizer_create) create_fn;
    typedef decltype(&lpq_search) search_fn;
    typedef decltype(&lpq_search_workspace_bytes) ws_fn;
    typedef decltype(&lpq_last_error) err_fn;
    create_fn qcreate = (create_fn)dlsym(lib, "lpq_quantizer_create");
    search_fn search = (search_fn)dlsym(lib, "lpq_search");
    ws_fn wsb = (ws_fn)dlsym(lib, "lpq_search_workspace_bytes");
    err_fn last = (err_fn)dlsym(lib, "lpq_last_error");
    CHECK(qcreate && search && wsb && last, "symbols");
    if (!(qcreate && search && wsb && last)) return;
    lpq_quantizer *h = nullptr;
    CHECK(qcreate(nullptr, 8, 8) == 1, "null out");
    CHECK(qcreate(&h, 0, 8) == 1 && h == nullptr, "d = 0");
    CHECK(qcreate(&h, 8, 0) == 1 && h == nullptr, "bits = 0");
    CHECK(last()[0] != 0, "message set");
    CHECK(search(nullptr, nullptr, 1, 1, 1, 0, nullptr, nullptr, nullptr, 0, nullptr) == 1, "null index");
    CHECK(wsb(nullptr, 10, 10, 0) == 0, "null index has no workspace size");
    printf("abi: argument checks passed\n");
}

int main(int argc, char **argv)
{
    oracle_checks();
    if (argc > 1) {
        void *lib = dlopen(argv[1], RTLD_NOW | RTLD_LOCAL);
        if (!lib) { printf("dlopen %s: %s\n", argv[1], dlerror()); return 2; }
        planner_checks(lib);
        abi_checks(lib);
    }
    if (g_fail) { printf("%d check(s) failed\n", g_fail); return 1; }
    printf("all host checks passed\n");
    return 0;
}
