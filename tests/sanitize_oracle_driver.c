/* Drives every entry point of the CPU oracle (oracle/rps_oracle.c) over shapes that reach its
 * edges -- one worker, 64 workers, a single column per block, sampled columns past 2^32, bf16
 * storage, external servers whose uplinks are all lost -- in a program built with
 * -fsanitize=address,undefined (tests/test_sanitizers.py).  Prints a checksum per case; the test
 * compares them with the regular build of the oracle, so the instrumented run also has to
 * compute the same values. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

void rps_oracle_philox4x32(uint32_t rounds, const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
void rps_oracle_masks(uint64_t seed, uint64_t step, int32_t n, int32_t nb, double p, int32_t server_mode,
                      int32_t *server, uint8_t *U, uint8_t *D);
float rps_oracle_noise_radius(uint32_t kr);
void rps_oracle_noise_direction(uint32_t ka, float *c, float *s);
void rps_oracle_noise_patch(uint64_t seed, uint64_t step, int32_t pair, uint64_t quad, float sigma, float out[8]);
float rps_oracle_noise(uint64_t seed, uint64_t step, int32_t worker, int64_t column, float sigma);
void rps_oracle_local_step(void *X, const void *G, int32_t n, int64_t m, const int64_t *cols, int32_t dtype,
                           float gamma, float sigma, float lambda, uint64_t seed, uint64_t step, int32_t threads);
void rps_oracle_lossy_average(void *V, int32_t n, int64_t m, const int64_t *cols, int32_t nb, const int64_t *offsets,
                              const uint8_t *U, const uint8_t *D, int32_t dtype, int32_t threads);
void rps_oracle_build_W(int32_t n, int32_t nb, int32_t j, const uint8_t *U, const uint8_t *D, double *W);
int32_t rps_oracle_max_threads(void);

static uint64_t mix(uint64_t h, const void *data, size_t bytes)
{
    const unsigned char *p = (const unsigned char *)data;
    for (size_t k = 0; k < bytes; ++k) { h ^= p[k]; h *= 1099511628211ull; }
    return h;
}

static void fill(float *x, int64_t count, uint32_t salt)
{
    for (int64_t k = 0; k < count; ++k) {
        uint32_t ctr[4] = { (uint32_t)k, (uint32_t)(k >> 32), salt, 77u }, key[2] = { 1u, 2u }, w[4];
        rps_oracle_philox4x32(10, ctr, key, w);
        x[k] = ((float)(w[0] >> 8) - 8388608.0f) * (1.0f / 8388608.0f);
    }
}

static uint16_t to_bf16(float f)
{
    uint32_t u; memcpy(&u, &f, 4);
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

/* one round on [n, m] with nb blocks; cols == NULL or sampled model coordinates */
static uint64_t round_case(int32_t n, int64_t m, int32_t nb, int32_t mode, int32_t dtype, double p, const int64_t *cols,
                           const int64_t *offsets, int with_g, int32_t threads)
{
    uint64_t h = 1469598103934665603ull;
    const size_t elem = dtype == 0 ? 4 : 2;
    float *xf = (float *)malloc((size_t)(n * m) * sizeof(float));
    float *gf = (float *)malloc((size_t)(n * m) * sizeof(float));
    void *X = malloc((size_t)(n * m) * elem), *G = malloc((size_t)(n * m) * elem);
    int32_t *server = (int32_t *)malloc((size_t)nb * sizeof(int32_t));
    uint8_t *U = (uint8_t *)malloc((size_t)(n * nb)), *D = (uint8_t *)malloc((size_t)(n * nb));
    double *W = (double *)malloc((size_t)(n * n) * sizeof(double));
    fill(xf, n * m, 1u); fill(gf, n * m, 2u);
    for (int64_t k = 0; k < n * m; ++k) {
        if (dtype == 0) { ((float *)X)[k] = xf[k]; ((float *)G)[k] = gf[k]; }
        else { ((uint16_t *)X)[k] = to_bf16(xf[k]); ((uint16_t *)G)[k] = to_bf16(gf[k]); }
    }
    for (uint64_t step = 0; step < 3; ++step) {
        const uint64_t t = step == 2 ? ((1ull << 56) - 1) : step;
        rps_oracle_local_step(X, with_g ? G : NULL, n, m, cols, dtype, 0.25f, 0.5f, 0.01f, 42u, t, threads);
        rps_oracle_masks(42u, t, n, nb, p, mode, server, U, D);
        rps_oracle_lossy_average(X, n, m, cols, nb, offsets, U, D, dtype, threads);
        h = mix(h, server, (size_t)nb * sizeof(int32_t));
        h = mix(h, U, (size_t)(n * nb)); h = mix(h, D, (size_t)(n * nb));
        h = mix(h, X, (size_t)(n * m) * elem);
    }
    for (int32_t j = 0; j < nb; j += (nb > 3 ? nb / 3 : 1)) {
        rps_oracle_build_W(n, nb, j, U, D, W);
        double colsum = 0.0;
        for (int32_t k = 0; k < n * n; ++k) colsum += W[k];
        if (fabs(colsum - (double)n) > 1e-9) { fprintf(stderr, "W is not column-stochastic\n"); exit(3); }
    }
    free(xf); free(gf); free(X); free(G); free(server); free(U); free(D); free(W);
    return h;
}

int main(void)
{
    /* hash, noise cells, noise indexing at the ends of the counter range */
    uint64_t h = 1469598103934665603ull;
    for (uint32_t k = 0; k < 4096; k += 97) {
        float c, s, r = rps_oracle_noise_radius(k);
        rps_oracle_noise_direction(k, &c, &s);
        h = mix(h, &r, 4); h = mix(h, &c, 4); h = mix(h, &s, 4);
    }
    float patch[8];
    rps_oracle_noise_patch(~0ull, (1ull << 56) - 1, 31, (1ull << 32) - 1, 0.1f, patch);
    h = mix(h, patch, sizeof patch);
    float z = rps_oracle_noise(7u, 9u, 63, (1ll << 34) - 1, 1.0f);
    h = mix(h, &z, 4);
    printf("noise %016llx\n", (unsigned long long)h);

    int64_t off1[2] = { 0, 37 };
    printf("n1 %016llx\n", (unsigned long long)round_case(1, 37, 1, 0, 0, 0.5, NULL, off1, 0, 1));

    int64_t off64[65];
    for (int j = 0; j <= 64; ++j) off64[j] = j;                       /* one column per block */
    printf("n64_single_columns %016llx\n", (unsigned long long)round_case(64, 64, 64, 0, 0, 0.1, NULL, off64, 1, 2));

    int64_t off5[6] = { 0, 1, 400, 401, 999, 1003 };                  /* ragged blocks, bf16, identity servers */
    printf("n5_bf16 %016llx\n", (unsigned long long)round_case(5, 1003, 5, 1, 1, 0.3, NULL, off5, 0, 3));

    int64_t offbig[4] = { 0, (1ll << 32) + 5, (1ll << 33), (1ll << 34) };   /* sampled columns of a 2^34-wide model */
    int64_t cols[8] = { 0, 3, (1ll << 32) + 4, (1ll << 32) + 5, (1ll << 33) - 1, (1ll << 33), (1ll << 34) - 2, (1ll << 34) - 1 };
    printf("sampled_wide %016llx\n", (unsigned long long)round_case(3, 8, 3, 0, 1, 0.4, cols, offbig, 0, 2));

    int64_t offext[3] = { 0, 100, 257 };                               /* external servers, every uplink lost */
    printf("external_p1 %016llx\n", (unsigned long long)round_case(6, 257, 2, 2, 0, 1.0, NULL, offext, 1, 1));
    printf("external %016llx\n", (unsigned long long)round_case(6, 257, 2, 2, 0, 0.6, NULL, offext, 0, 1));
    printf("threads %d\n", (int)rps_oracle_max_threads() > 0);
    return 0;
}
