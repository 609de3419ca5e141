/* The C ABI used from plain C (gcc, C99): builds a small model with spdnn_create, runs
 * spdnn_infer and checks the result against a closed form of Eq. 1 (Section II-A-1).
 *
 * The same inference is then repeated through spdnn_infer_static (no work arena) and spdnn_infer_host
 * (inputs in host memory, in batches of two rows).
 *
 * Model: N neurons, L layers, neuron j connected to columns (j + 3k) mod N, k = 0..31, all
 * weights 1/16, bias -0.25.  A row of constant c then maps to the constant
 * min(max(2c - 0.25, 0), 32) whatever the pattern (32 weights of 1/16 sum to 2, and all the
 * products are exact in float).  Rows: c = 0 (dropped after the first layer), 0.1 (2c - 0.25 < 0:
 * dropped), 1 (grows to the clip), 20 (clipped at once).
 *
 * Prints "c abi ok" and exits 0 on success; test infrastructure, built by the package's build
 * step, run by tests/test_gpu_c_abi.py. */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <math.h>
#include <stdio.h>
#include <stdlib.h>

#include "../../include/spdnn.h"

#define CHECK_HIP(x)                                                                  \
    do {                                                                              \
        hipError_t e_ = (x);                                                          \
        if (e_ != hipSuccess) {                                                       \
            fprintf(stderr, "%s failed: %s\n", #x, hipGetErrorString(e_));            \
            return 2;                                                                 \
        }                                                                             \
    } while (0)
#define CHECK_SP(x)                                                                   \
    do {                                                                              \
        int rc_ = (x);                                                                \
        if (rc_ != SPDNN_OK) {                                                        \
            fprintf(stderr, "%s failed (%d): %s\n", #x, rc_, spdnn_last_error());     \
            return 3;                                                                 \
        }                                                                             \
    } while (0)

int main(void) {
    enum { N = 2052, L = 5, BATCH = 4 };
    const float consts[BATCH] = {0.0f, 0.1f, 1.0f, 20.0f};
    int32_t* idx[L];
    float* val[L];
    float* bias = (float*)malloc(sizeof(float) * N);
    float* y0 = (float*)malloc(sizeof(float) * BATCH * N);
    int l, j, k, r;
    for (l = 0; l < L; ++l) {
        idx[l] = (int32_t*)malloc(sizeof(int32_t) * N * 32);
        val[l] = (float*)malloc(sizeof(float) * N * 32);
        for (j = 0; j < N; ++j)
            for (k = 0; k < 32; ++k) {
                idx[l][j * 32 + k] = (j + 3 * k + l) % N;
                val[l][j * 32 + k] = 0.0625f;
            }
    }
    for (j = 0; j < N; ++j) bias[j] = -0.25f;
    for (r = 0; r < BATCH; ++r)
        for (j = 0; j < N; ++j) y0[r * N + j] = consts[r];

    size_t wbytes = 0, kbytes = 0;
    CHECK_SP(spdnn_weights_bytes(N, L, &wbytes));
    CHECK_SP(spdnn_work_bytes(N, BATCH, &kbytes));
    void *warena = NULL, *karena = NULL, *y0_dev = NULL, *rows_dev = NULL, *yf_dev = NULL;
    CHECK_HIP(hipMalloc(&warena, wbytes));
    CHECK_HIP(hipMalloc(&karena, kbytes));
    CHECK_HIP(hipMalloc(&y0_dev, sizeof(float) * BATCH * N));
    CHECK_HIP(hipMalloc(&rows_dev, sizeof(int32_t) * BATCH));
    CHECK_HIP(hipMalloc(&yf_dev, sizeof(float) * BATCH * N));
    CHECK_HIP(hipMemcpy(y0_dev, y0, sizeof(float) * BATCH * N, hipMemcpyHostToDevice));

    spdnn_t net = NULL;
    CHECK_SP(spdnn_create(&net, N, L, (const int32_t* const*)idx, (const float* const*)val, bias, SPDNN_HOST, warena,
                          wbytes, NULL));
    int32_t n_active = -1;
    CHECK_SP(spdnn_infer(net, (const float*)y0_dev, BATCH, karena, kbytes, &n_active, (int32_t*)rows_dev,
                         (float*)yf_dev));

    /* closed form: iterate c -> min(max(2c - 0.25, 0), 32) in float, as the library does */
    int32_t want_rows[BATCH];
    float want_val[BATCH];
    int want_n = 0;
    for (r = 0; r < BATCH; ++r) {
        float c = consts[r];
        int alive = 1;
        for (l = 0; l < L && alive; ++l) {
            float z = 2.0f * c + -0.25f;
            c = z < 0.0f ? 0.0f : z > 32.0f ? 32.0f : z;
            alive = c > 0.0f;
        }
        if (alive) {
            want_rows[want_n] = r;
            want_val[want_n] = c;
            ++want_n;
        }
    }
    if (n_active != want_n) {
        fprintf(stderr, "n_active = %d, expected %d\n", (int)n_active, want_n);
        return 1;
    }
    int32_t rows[BATCH];
    float* yf = (float*)malloc(sizeof(float) * BATCH * N);
    CHECK_HIP(hipMemcpy(rows, rows_dev, sizeof(int32_t) * (size_t)want_n, hipMemcpyDeviceToHost));
    CHECK_HIP(hipMemcpy(yf, yf_dev, sizeof(float) * (size_t)want_n * N, hipMemcpyDeviceToHost));
    for (r = 0; r < want_n; ++r) {
        if (rows[r] != want_rows[r]) {
            fprintf(stderr, "active row %d is %d, expected %d\n", r, (int)rows[r], (int)want_rows[r]);
            return 1;
        }
        for (j = 0; j < N; ++j)
            if (fabsf(yf[r * N + j] - want_val[r]) > 1e-5f * want_val[r]) {
                fprintf(stderr, "row %d neuron %d: %g, expected %g\n", (int)rows[r], j, (double)yf[r * N + j],
                        (double)want_val[r]);
                return 1;
            }
    }
    /* the same inference without a work arena (static scratch) and with the inputs left in host memory,
     * two rows at a time: same rows, same values */
    {
        int32_t n2 = -1, rows2[BATCH];
        int which;
        size_t hbytes = 0;
        void* harena = NULL;
        CHECK_SP(spdnn_host_work_bytes(N, 2, &hbytes));
        CHECK_HIP(hipMalloc(&harena, hbytes));
        for (which = 0; which < 2; ++which) {
            CHECK_HIP(hipMemset(rows_dev, 0xff, sizeof(int32_t) * BATCH));
            CHECK_HIP(hipMemset(yf_dev, 0xff, sizeof(float) * BATCH * N));
            if (which == 0)
                CHECK_SP(spdnn_infer_static(net, (const float*)y0_dev, BATCH, &n2, (int32_t*)rows_dev, (float*)yf_dev));
            else
                CHECK_SP(spdnn_infer_host(net, y0, BATCH, 2, harena, hbytes, &n2, (int32_t*)rows_dev, (float*)yf_dev));
            if (n2 != want_n) {
                fprintf(stderr, "entry point %d: n_active = %d, expected %d\n", which, (int)n2, want_n);
                return 1;
            }
            CHECK_HIP(hipMemcpy(rows2, rows_dev, sizeof(int32_t) * (size_t)want_n, hipMemcpyDeviceToHost));
            CHECK_HIP(hipMemcpy(yf, yf_dev, sizeof(float) * (size_t)want_n * N, hipMemcpyDeviceToHost));
            for (r = 0; r < want_n; ++r) {
                if (rows2[r] != want_rows[r]) {
                    fprintf(stderr, "entry point %d: active row %d is %d, expected %d\n", which, r, (int)rows2[r],
                            (int)want_rows[r]);
                    return 1;
                }
                for (j = 0; j < N; ++j)
                    if (fabsf(yf[r * N + j] - want_val[r]) > 1e-5f * want_val[r]) {
                        fprintf(stderr, "entry point %d: row %d neuron %d: %g, expected %g\n", which, (int)rows2[r], j,
                                (double)yf[r * N + j], (double)want_val[r]);
                        return 1;
                    }
            }
        }
        hipFree(harena);
    }
    int32_t kind = -1, passes = -1, one = -1;
    CHECK_SP(spdnn_layer_kernel(net, 0, &kind));
    CHECK_SP(spdnn_layer_passes(net, 0, &passes));
    CHECK_SP(spdnn_one_launch(net, BATCH, &one));
    if (one != 0 && one != 1) {
        fprintf(stderr, "spdnn_one_launch answered %d\n", one);
        return 1;
    }
    CHECK_SP(spdnn_destroy(net));
    /* error path: a positive bias must be refused */
    bias[5] = 0.5f;
    if (spdnn_create(&net, N, L, (const int32_t* const*)idx, (const float* const*)val, bias, SPDNN_HOST, warena, wbytes,
                     NULL) != SPDNN_EBIAS || net != NULL) {
        fprintf(stderr, "positive bias was not refused\n");
        return 1;
    }
    printf("c abi ok: %d of %d rows active, values %g and %g, layer 0 on kernel %d in %d pass\n", (int)n_active, BATCH,
           (double)want_val[0], (double)want_val[want_n - 1], (int)kind, (int)passes);
    hipFree(warena);
    hipFree(karena);
    hipFree(y0_dev);
    hipFree(rows_dev);
    hipFree(yf_dev);
    return 0;
}
