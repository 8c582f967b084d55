// Context measurement for bench.py --vendor-compare (not on the product path, not linked into libquartet.so):
// the MXFP4 GEMM of the vendor library (hipBLASLt: E2M1 operands, one E8M0 scale per 32 along K, fp32 result)
// and quartet_mxfp4_gemm on the same device buffers, shapes and random codes, timed with HIP events.
// Usage: vendor_mxfp4_gemm <path to libquartet.so> m n k [m n k ...]; prints one JSON object per shape.
#include <dlfcn.h>
#include <hip/hip_runtime.h>
#include <hipblaslt/hipblaslt.h>

#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <vector>

#define CHECK(x)                                                                        \
    do {                                                                                \
        auto e_ = (x);                                                                  \
        if (e_ != 0) {                                                                  \
            fprintf(stderr, "%s failed with %d (line %d)\n", #x, (int)e_, __LINE__);    \
            return 1;                                                                   \
        }                                                                               \
    } while (0)

typedef int (*gemm_fn)(const uint8_t*, const uint8_t*, const uint8_t*, const uint8_t*, int64_t, int64_t, int64_t, float,
                       void*, int, int64_t, void*);
typedef size_t (*scale_bytes_fn)(int64_t, int64_t);

static int time_ms(float* out, int reps, int (*call)(void*), void* ctx) {
    for (int i = 0; i < 3; ++i) CHECK(call(ctx));
    CHECK(hipDeviceSynchronize());
    hipEvent_t e0, e1;
    CHECK(hipEventCreate(&e0));
    CHECK(hipEventCreate(&e1));
    CHECK(hipEventRecord(e0, 0));
    for (int i = 0; i < reps; ++i) CHECK(call(ctx));
    CHECK(hipEventRecord(e1, 0));
    CHECK(hipDeviceSynchronize());
    CHECK(hipEventElapsedTime(out, e0, e1));
    *out /= reps;
    CHECK(hipEventDestroy(e0));
    CHECK(hipEventDestroy(e1));
    return 0;
}

struct Ctx {
    hipblasLtHandle_t h;
    hipblasLtMatmulDesc_t desc;
    hipblasLtMatrixLayout_t la, lb, lc;
    hipblasLtMatmulAlgo_t algo;
    void *a, *b, *d, *ws;
    size_t ws_bytes;
    gemm_fn ours;
    const uint8_t *sa, *sb;
    int64_t m, n, k;
};

static int call_vendor(void* p) {
    Ctx* c = (Ctx*)p;
    const float alpha = 1.0f, beta = 0.0f;
    return (int)hipblasLtMatmul(c->h, c->desc, &alpha, c->a, c->la, c->b, c->lb, &beta, c->d, c->lc, c->d, c->lc, &c->algo, c->ws,
                                c->ws_bytes, 0);
}
static int call_ours(void* p) {
    Ctx* c = (Ctx*)p;
    return c->ours((const uint8_t*)c->a, c->sa, (const uint8_t*)c->b, c->sb, c->m, c->n, c->k, 1.0f, c->d, 0, c->n, nullptr);
}

int main(int argc, char** argv) {
    if (argc < 5 || (argc - 2) % 3 != 0) {
        fprintf(stderr, "usage: %s libquartet.so m n k [m n k ...]\n", argv[0]);
        return 2;
    }
    void* lib = dlopen(argv[1], RTLD_NOW);
    if (!lib) {
        fprintf(stderr, "cannot load %s\n", argv[1]);
        return 2;
    }
    gemm_fn ours = (gemm_fn)dlsym(lib, "quartet_mxfp4_gemm");
    scale_bytes_fn scale_bytes = (scale_bytes_fn)dlsym(lib, "quartet_scale_bytes");
    if (!ours || !scale_bytes) return 2;
    Ctx c = {};
    c.ours = ours;
    CHECK(hipblasLtCreate(&c.h));
    c.ws_bytes = (size_t)256 << 20;
    CHECK(hipMalloc(&c.ws, c.ws_bytes));
    for (int s = 2; s + 2 < argc; s += 3) {
        const int64_t m = atoll(argv[s]), n = atoll(argv[s + 1]), k = atoll(argv[s + 2]);
        c.m = m; c.n = n; c.k = k;
        const size_t sa_bytes = scale_bytes(m, k), sb_bytes = scale_bytes(n, k);
        uint8_t *sa, *sb;
        CHECK(hipMalloc(&c.a, m * k / 2));
        CHECK(hipMalloc(&c.b, n * k / 2));
        CHECK(hipMalloc(&sa, sa_bytes));
        CHECK(hipMalloc(&sb, sb_bytes));
        CHECK(hipMalloc(&c.d, m * n * 4));
        c.sa = sa; c.sb = sb;
        // uniformly random codes, scale bytes 120..133 (no infinities): the data the GEMM sweeps of this repository use
        std::vector<uint8_t> host(m * k / 2 > n * k / 2 ? m * k / 2 : n * k / 2);
        uint32_t rng = 12345u + (uint32_t)s;
        auto next = [&]() { rng = rng * 1664525u + 1013904223u; return (uint8_t)(rng >> 24); };
        for (auto& v : host) v = next();
        CHECK(hipMemcpy(c.a, host.data(), m * k / 2, hipMemcpyHostToDevice));
        for (auto& v : host) v = next();
        CHECK(hipMemcpy(c.b, host.data(), n * k / 2, hipMemcpyHostToDevice));
        std::vector<uint8_t> hs(sa_bytes > sb_bytes ? sa_bytes : sb_bytes);
        for (auto& v : hs) v = (uint8_t)(120 + next() % 14);
        CHECK(hipMemcpy(sa, hs.data(), sa_bytes, hipMemcpyHostToDevice));
        CHECK(hipMemcpy(sb, hs.data(), sb_bytes, hipMemcpyHostToDevice));

        CHECK(hipblasLtMatmulDescCreate(&c.desc, HIPBLAS_COMPUTE_32F, HIP_R_32F));
        hipblasOperation_t ta = HIPBLAS_OP_T, tb = HIPBLAS_OP_N;
        CHECK(hipblasLtMatmulDescSetAttribute(c.desc, HIPBLASLT_MATMUL_DESC_TRANSA, &ta, sizeof(ta)));
        CHECK(hipblasLtMatmulDescSetAttribute(c.desc, HIPBLASLT_MATMUL_DESC_TRANSB, &tb, sizeof(tb)));
        hipblasLtMatmulMatrixScale_t mode = HIPBLASLT_MATMUL_MATRIX_SCALE_VEC32_UE8M0;
        CHECK(hipblasLtMatmulDescSetAttribute(c.desc, HIPBLASLT_MATMUL_DESC_A_SCALE_MODE, &mode, sizeof(mode)));
        CHECK(hipblasLtMatmulDescSetAttribute(c.desc, HIPBLASLT_MATMUL_DESC_B_SCALE_MODE, &mode, sizeof(mode)));
        CHECK(hipblasLtMatmulDescSetAttribute(c.desc, HIPBLASLT_MATMUL_DESC_A_SCALE_POINTER, &sa, sizeof(sa)));
        CHECK(hipblasLtMatmulDescSetAttribute(c.desc, HIPBLASLT_MATMUL_DESC_B_SCALE_POINTER, &sb, sizeof(sb)));
        // the library is column-major: both operands K-contiguous = A^T (k x m, lda = k) times B (k x n, ldb = k)
        CHECK(hipblasLtMatrixLayoutCreate(&c.la, HIP_R_4F_E2M1, k, m, k));
        CHECK(hipblasLtMatrixLayoutCreate(&c.lb, HIP_R_4F_E2M1, k, n, k));
        CHECK(hipblasLtMatrixLayoutCreate(&c.lc, HIP_R_32F, m, n, m));
        hipblasLtMatmulPreference_t pref;
        CHECK(hipblasLtMatmulPreferenceCreate(&pref));
        CHECK(hipblasLtMatmulPreferenceSetAttribute(pref, HIPBLASLT_MATMUL_PREF_MAX_WORKSPACE_BYTES, &c.ws_bytes, sizeof(c.ws_bytes)));
        hipblasLtMatmulHeuristicResult_t res[4];
        int found = 0;
        CHECK(hipblasLtMatmulAlgoGetHeuristic(c.h, c.desc, c.la, c.lb, c.lc, c.lc, pref, 4, res, &found));
        float best = 0.0f;
        for (int al = 0; al < found; ++al) {      // best of the heuristic's first algorithms
            c.algo = res[al].algo;
            float ms = 0.0f;
            if (time_ms(&ms, 10, call_vendor, &c)) return 1;
            if (best == 0.0f || ms < best) best = ms;
        }
        float mine = 0.0f;
        if (time_ms(&mine, 10, call_ours, &c)) return 1;
        const double flop = 2.0 * (double)m * (double)n * (double)k;
        printf("{\"m\": %lld, \"n\": %lld, \"k\": %lld, \"vendor_algorithms\": %d, \"vendor_ms\": %.4f, \"vendor_tflops\": %.1f, "
               "\"quartet_ms\": %.4f, \"quartet_tflops\": %.1f}\n",
               (long long)m, (long long)n, (long long)k, found, best, best > 0 ? flop / best / 1e9 : 0.0, mine, flop / mine / 1e9);
        fflush(stdout);
        CHECK(hipblasLtMatmulPreferenceDestroy(pref));
        CHECK(hipblasLtMatrixLayoutDestroy(c.la));
        CHECK(hipblasLtMatrixLayoutDestroy(c.lb));
        CHECK(hipblasLtMatrixLayoutDestroy(c.lc));
        CHECK(hipblasLtMatmulDescDestroy(c.desc));
        CHECK(hipFree(c.a)); CHECK(hipFree(c.b)); CHECK(hipFree(sa)); CHECK(hipFree(sb)); CHECK(hipFree(c.d));
    }
    return 0;
}
