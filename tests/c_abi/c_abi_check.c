/*
 * The C ABI of libbiq used from plain C: no Python, no torch, only the HIP runtime for device
 * memory.  Packs random signs, runs biq_gemm with the library's own plan for three shapes (GEMV,
 * batched tables, matrix cores) and compares with the CPU oracle (linked from oracle/).
 * Test infrastructure: built by the repository's build step, run by tests/test_c_abi.py.
 */
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "biq.h"

int biqo_gemm_dense(const int8_t* B, const float* alpha, const float* X, long m, long n, int q, long b,
                    double* Y);

#define CHECK_HIP(x)                                                              \
    do {                                                                          \
        hipError_t e_ = (x);                                                      \
        if (e_ != hipSuccess) {                                                   \
            fprintf(stderr, "HIP error %d at %s:%d\n", (int)e_, __FILE__, __LINE__); \
            return 2;                                                             \
        }                                                                         \
    } while (0)
#define CHECK_BIQ(x)                                                                         \
    do {                                                                                     \
        biq_status s_ = (x);                                                                 \
        if (s_ != BIQ_OK) {                                                                  \
            fprintf(stderr, "libbiq: %s at %s:%d\n", biq_status_str(s_), __FILE__, __LINE__); \
            return 3;                                                                        \
        }                                                                                    \
    } while (0)

static uint64_t rng_state = 0x2005099040ull;
static uint32_t rng_next(void) {  /* xorshift64* */
    rng_state ^= rng_state >> 12;
    rng_state ^= rng_state << 25;
    rng_state ^= rng_state >> 27;
    return (uint32_t)((rng_state * 0x2545F4914F6CDD1Dull) >> 32);
}
static float rng_unit(void) { return (float)(rng_next() >> 8) / 16777216.0f; }

static int run_case(int m, int n, int q, int batch, int mu) {
    const size_t nB = (size_t)q * m * n, nA = (size_t)q * m, nX = (size_t)batch * n, nY = (size_t)batch * m;
    int8_t* B = (int8_t*)malloc(nB);
    float* alpha = (float*)malloc(nA * sizeof(float));
    float* X = (float*)malloc(nX * sizeof(float));
    float* Y = (float*)malloc(nY * sizeof(float));
    double* ref = (double*)malloc(nY * sizeof(double));
    if (!B || !alpha || !X || !Y || !ref) return 4;
    for (size_t i = 0; i < nB; ++i) B[i] = (rng_next() & 1u) ? 1 : -1;
    for (size_t i = 0; i < nA; ++i) alpha[i] = 0.05f + 0.95f * rng_unit();
    for (size_t i = 0; i < nX; ++i) X[i] = 2.0f * rng_unit() - 1.0f;

    biq_plan plan;
    CHECK_BIQ(biq_plan_get(m, n, q, batch, mu, &plan));
    const size_t kbytes = biq_packed_bytes(m, n, q), wbytes = biq_workspace_bytes(m, n, q, batch, mu);
    void *dB, *dK, *dA, *dX, *dY, *dW = NULL;
    CHECK_HIP(hipMalloc(&dB, nB));
    CHECK_HIP(hipMalloc(&dK, kbytes));
    CHECK_HIP(hipMalloc(&dA, nA * sizeof(float)));
    CHECK_HIP(hipMalloc(&dX, nX * sizeof(float)));
    CHECK_HIP(hipMalloc(&dY, nY * sizeof(float)));
    if (wbytes) CHECK_HIP(hipMalloc(&dW, wbytes));
    CHECK_HIP(hipMemcpy(dB, B, nB, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dA, alpha, nA * sizeof(float), hipMemcpyHostToDevice));
    CHECK_HIP(hipMemcpy(dX, X, nX * sizeof(float), hipMemcpyHostToDevice));
    hipStream_t stream;
    CHECK_HIP(hipStreamCreate(&stream));
    CHECK_BIQ(biq_pack((const int8_t*)dB, (uint8_t*)dK, m, n, q, mu, stream));
    CHECK_BIQ(biq_gemm((const uint8_t*)dK, (const float*)dA, (const float*)dX, (float*)dY, m, n, q, batch, mu,
                       dW, wbytes, stream));
    CHECK_HIP(hipStreamSynchronize(stream));
    CHECK_HIP(hipMemcpy(Y, dY, nY * sizeof(float), hipMemcpyDeviceToHost));

    if (biqo_gemm_dense(B, alpha, X, m, n, q, batch, ref) != 0) return 5;
    /* the stated bar: per input vector max|dy| <= 1e-4 * max_r sum_i |alpha_i[r]| * ||x||_1 */
    double amax = 0.0;
    for (int r = 0; r < m; ++r) {
        double s = 0.0;
        for (int i = 0; i < q; ++i) s += fabs((double)alpha[(size_t)i * m + r]);
        if (s > amax) amax = s;
    }
    int bad = 0;
    double worst = 0.0;
    for (int a = 0; a < batch; ++a) {
        double l1 = 0.0;
        for (int j = 0; j < n; ++j) l1 += fabs((double)X[(size_t)a * n + j]);
        for (int r = 0; r < m; ++r) {
            const double d = fabs((double)Y[(size_t)a * m + r] - ref[(size_t)a * m + r]);
            if (d > worst) worst = d;
            if (!(d <= 1e-4 * amax * l1)) ++bad;
        }
    }
    printf("m=%d n=%d q=%d batch=%d mu=%d kernel=%s max|dy|=%.3e %s\n", m, n, q, batch, mu,
           biq_kernel_name(plan.kernel), worst, bad ? "FAIL" : "ok");
    hipFree(dB); hipFree(dK); hipFree(dA); hipFree(dX); hipFree(dY); if (dW) hipFree(dW);
    hipStreamDestroy(stream);
    free(B); free(alpha); free(X); free(Y); free(ref);
    return bad ? 1 : 0;
}

int main(void) {
    printf("libbiq version %d\n", biq_version());
    int rc = 0;
    rc |= run_case(777, 2048, 2, 1, 8);      /* GEMV, half tables */
    rc |= run_case(500, 1000, 3, 6, 8);      /* batched tables */
    rc |= run_case(300, 2100, 2, 3, 4);      /* narrow keys */
    rc |= run_case(4096, 2048, 2, 96, 8);    /* matrix cores */
    printf(rc ? "C ABI check FAILED\n" : "C ABI check passed\n");
    return rc;
}
