/* Calls the host-only paths of the HIP library's C ABI (argument validation, size helpers, the
 * noise-cell table, error strings) from a program built with -fsanitize=address,undefined against
 * a copy of the library whose C-ABI translation unit is built with the same host sanitizers
 * (tests/test_sanitizers.py).  No GPU call is reached: every rps_create below fails validation. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "rps.h"

#define EXPECT(cond) do { if (!(cond)) { fprintf(stderr, "line %d: %s\n", __LINE__, #cond); return 1; } } while (0)

int main(void)
{
    rps_ctx *ctx = NULL;
    int64_t bad_off[5] = { 0, 10, 10, 50, 100 };
    EXPECT(rps_create(&ctx, 0, 100, NULL, 0.1, 0.1f, 0, RPS_DTYPE_F32, 0, NULL) == RPS_EINVAL);
    EXPECT(rps_create(&ctx, 65, 6500, NULL, 0.1, 0.1f, 0, RPS_DTYPE_F32, 0, NULL) == RPS_EINVAL);
    EXPECT(rps_create(&ctx, 4, 101, NULL, 0.1, 0.1f, 0, RPS_DTYPE_F32, 0, NULL) == RPS_EINVAL);
    EXPECT(rps_create(&ctx, 4, 100, NULL, nan(""), 0.1f, 0, RPS_DTYPE_F32, 0, NULL) == RPS_EINVAL);
    EXPECT(rps_create(&ctx, 4, 100, NULL, 0.1, INFINITY, 0, RPS_DTYPE_F32, 0, NULL) == RPS_EINVAL);
    EXPECT(rps_create(&ctx, 4, 100, NULL, 0.1, 0.1f, 0, 7, 0, NULL) == RPS_EINVAL);
    EXPECT(rps_create(&ctx, 4, 100, NULL, 0.1, 0.1f, 0, RPS_DTYPE_F32, 64u, NULL) == RPS_EINVAL);
    EXPECT(rps_create(&ctx, 4, 100, bad_off, 0.1, 0.1f, 0, RPS_DTYPE_F32, 0, NULL) == RPS_EINVAL);
    EXPECT(rps_create(NULL, 4, 100, NULL, 0.1, 0.1f, 0, RPS_DTYPE_F32, 0, NULL) == RPS_EINVAL);
    EXPECT(rps_create_external(&ctx, 4, 0, 100, NULL, 0.1, 0.1f, 0, RPS_DTYPE_F32, NULL) == RPS_EINVAL);
    EXPECT(ctx == NULL);
    EXPECT(rps_destroy(NULL) == RPS_OK);
    EXPECT(rps_local_step(NULL, NULL, NULL, 0) == RPS_EINVAL);
    EXPECT(rps_lossy_average(NULL, NULL, 0) == RPS_EINVAL);
    EXPECT(rps_round(NULL, NULL, NULL, 0) == RPS_EINVAL);
    EXPECT(rps_round_gradient_averaging(NULL, NULL, NULL, 0) == RPS_EINVAL);
    EXPECT(rps_set_gamma(NULL, 0.1f) == RPS_EINVAL);
    EXPECT(rps_set_row_pitch(NULL, 10) == RPS_EINVAL);
    EXPECT(rps_set_synthetic_grad(NULL, 0.1f, 0.0f) == RPS_EINVAL);
    EXPECT(rps_consensus_static(NULL, 4, 64, RPS_DTYPE_F32, 0, NULL, NULL) == RPS_EINVAL);
    EXPECT(rps_storage_elems(4, 1000, RPS_DTYPE_F32, 0) == 4000);
    EXPECT(rps_storage_elems(4, 1000, RPS_DTYPE_BF16, RPS_FLAG_LAYOUT_TILED) == 16 * 4 * 64);
    EXPECT(rps_storage_elems(0, 1000, RPS_DTYPE_F32, 0) == -1);
    EXPECT(rps_recommended_row_pitch(1 << 22, RPS_DTYPE_F32) == (1 << 22) + 1024);
    EXPECT(rps_recommended_row_pitch(0, RPS_DTYPE_F32) == -1);
    float *radius = (float *)malloc(4096 * sizeof(float)), *cs = (float *)malloc(8192 * sizeof(float));
    EXPECT(rps_noise_cells(radius, cs) == RPS_OK);
    EXPECT(rps_noise_cells(NULL, cs) == RPS_EINVAL);
    double sum = 0.0;
    for (int k = 0; k < 4096; ++k) sum += (double)cs[2 * k] * cs[2 * k] + (double)cs[2 * k + 1] * cs[2 * k + 1];
    EXPECT(fabs(sum - 4096.0) < 1e-3 && radius[0] > 4.24f && radius[4095] < 0.016f);
    free(radius); free(cs);
    /* host copy of the network-outcome generator: exact-size buffers at the smallest and largest shapes */
    for (int n = 1; n <= 64; n += 21) {
        const int servers[3] = { 0, 1, 64 };
        for (int k = 0; k < 3; ++k) {
            const int nb = servers[k] ? servers[k] : n;
            uint8_t *up = (uint8_t *)malloc((size_t)n * nb), *down = (uint8_t *)malloc((size_t)n * nb);
            int32_t *srv = (int32_t *)malloc((size_t)nb * sizeof(int32_t));
            EXPECT(rps_masks_host(n, servers[k], 0.25, 0x123456789abcdefULL, 0, (1ULL << 56) - 1, up, down, srv) == RPS_OK);
            EXPECT(rps_masks_host(n, servers[k], 1.0, 1, 0, 3, NULL, NULL, NULL) == RPS_OK);
            for (int j = 0; j < nb; ++j) EXPECT(servers[k] ? srv[j] == -1 : (srv[j] >= 0 && srv[j] < n && up[srv[j] * nb + j] == 1));
            free(up); free(down); free(srv);
        }
    }
    EXPECT(rps_masks_host(65, 0, 0.1, 0, 0, 0, NULL, NULL, NULL) == RPS_EINVAL);
    EXPECT(rps_masks_host(4, 0, 0.1, 0, 0, 1ULL << 56, NULL, NULL, NULL) == RPS_EINVAL);
    for (int code = 1; code >= -7; --code) EXPECT(rps_strerror(code) != NULL);
    EXPECT(rps_last_hip_error(NULL) == 0);
    printf("abi host paths ok\n");
    return 0;
}
