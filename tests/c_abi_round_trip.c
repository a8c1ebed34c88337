/* A plain C caller of the library (no Python, no PyTorch): device memory from the HIP runtime,
 * one context, three exact-averaging rounds (p = 0) and one lossy one, checked against what the
 * method fixes (Sec. 4.1: with every message delivered each block becomes the column mean of v;
 * with losses every receiver of a block holds the same bits).  Built and run by
 * tests/test_gpu_c_caller.py on the GPU. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include <hip/hip_runtime_api.h>

#include "rps.h"

#define CHECK(cond) do { if (!(cond)) { fprintf(stderr, "line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main(void)
{
    const int32_t n = 6;
    const int64_t N = 6 * 1000;
    const size_t bytes = (size_t)n * N * sizeof(float);
    float *host = (float *)malloc(bytes), *grad = (float *)malloc(bytes), *out = (float *)malloc(bytes);
    uint32_t s = 12345u;
    for (int64_t k = 0; k < n * N; ++k) {
        s = s * 1664525u + 1013904223u; host[k] = (float)(s >> 8) / 16777216.0f - 0.5f;
        s = s * 1664525u + 1013904223u; grad[k] = (float)(s >> 8) / 16777216.0f - 0.5f;
    }
    float *X = NULL, *G = NULL;
    CHECK(hipMalloc((void **)&X, bytes) == hipSuccess && hipMalloc((void **)&G, bytes) == hipSuccess);
    CHECK(hipMemcpy(X, host, bytes, hipMemcpyHostToDevice) == hipSuccess);
    CHECK(hipMemcpy(G, grad, bytes, hipMemcpyHostToDevice) == hipSuccess);

    rps_ctx *ctx = NULL;
    const float gamma = 0.25f;
    CHECK(rps_create(&ctx, n, N, NULL, 0.0, gamma, 7, RPS_DTYPE_F32, 0, NULL) == RPS_OK);
    CHECK(rps_round(ctx, X, G, 0) == RPS_OK);
    CHECK(hipDeviceSynchronize() == hipSuccess);
    CHECK(hipMemcpy(out, X, bytes, hipMemcpyDeviceToHost) == hipSuccess);
    double worst = 0.0;
    for (int64_t c = 0; c < N; ++c) {
        double mean = 0.0;
        for (int i = 0; i < n; ++i) mean += (double)fmaf(-gamma, grad[i * N + c], host[i * N + c]);
        mean /= n;
        for (int i = 0; i < n; ++i) {
            CHECK(out[i * N + c] == out[c]);   /* all workers identical after exact averaging */
            const double err = fabs((double)out[i * N + c] - mean);
            if (err > worst) worst = err;
        }
    }
    CHECK(worst < 1e-6);
    double dist = -1.0, msq = -1.0;
    CHECK(rps_consensus(ctx, X, &dist, &msq) == RPS_OK);
    CHECK(dist == 0.0 && msq > 0.0);
    CHECK(rps_destroy(ctx) == RPS_OK);

    /* lossy round: device masks equal the library's host copy; receivers of a block hold the same bits */
    CHECK(rps_create(&ctx, n, N, NULL, 0.4, gamma, 99, RPS_DTYPE_F32, 0, NULL) == RPS_OK);
    CHECK(hipMemcpy(X, host, bytes, hipMemcpyHostToDevice) == hipSuccess);
    uint8_t up[36], down[36], up_h[36], down_h[36];
    int32_t server[6], server_h[6];
    CHECK(rps_get_masks(ctx, 3, up, down, server) == RPS_OK);
    CHECK(rps_masks_host(n, 0, 0.4, 99, 0, 3, up_h, down_h, server_h) == RPS_OK);
    for (int k = 0; k < 36; ++k) CHECK(up[k] == up_h[k] && down[k] == down_h[k]);
    for (int j = 0; j < n; ++j) CHECK(server[j] == server_h[j]);
    CHECK(rps_local_step(ctx, X, G, 3) == RPS_OK);
    CHECK(rps_lossy_average(ctx, X, 3) == RPS_OK);
    CHECK(hipDeviceSynchronize() == hipSuccess);
    CHECK(hipMemcpy(out, X, bytes, hipMemcpyDeviceToHost) == hipSuccess);
    const int64_t width = N / n;
    for (int j = 0; j < n; ++j) {
        int first = -1;
        for (int i = 0; i < n; ++i) {
            if (!down[i * n + j]) {   /* reply lost: the worker keeps its own v */
                for (int64_t c = j * width; c < (j + 1) * width; ++c)
                    CHECK(out[i * N + c] == fmaf(-gamma, grad[i * N + c], host[i * N + c]));
                continue;
            }
            if (first < 0) { first = i; continue; }
            for (int64_t c = j * width; c < (j + 1) * width; ++c) CHECK(out[i * N + c] == out[first * N + c]);
        }
        CHECK(first >= 0);
    }
    CHECK(rps_destroy(ctx) == RPS_OK);
    CHECK(hipFree(X) == hipSuccess && hipFree(G) == hipSuccess);
    free(host); free(grad); free(out);
    printf("c caller ok\n");
    return 0;
}
