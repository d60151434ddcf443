/* Host-only driver that runs every oracle routine on small, ragged inputs.  It is compiled
 * together with oracle/core_oracle.c under AddressSanitizer and UndefinedBehaviorSanitizer by
 * tests/test_oracle_sanitizers.py; any out-of-bounds access or undefined operation aborts it. */
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <math.h>

void core_oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);
void core_oracle_xi_block(uint64_t seed, uint64_t round, uint32_t j, uint64_t q, double z[4]);
void core_oracle_xi_fill(uint64_t seed, uint64_t round, uint32_t j, uint64_t i0, uint64_t count, double *out);
int core_oracle_compress(uint64_t seed, uint64_t round, uint64_t d, uint32_t n, const void *G, int dtype,
                         uint64_t ld, const uint32_t *jidx, uint64_t nj, double *P);
int core_oracle_client_mean(const double *P, uint32_t n, uint64_t nj, double *pbar);
int core_oracle_reconstruct(uint64_t seed, uint64_t round, uint32_t m, const double *pbar, double scale,
                            uint64_t i0, uint64_t count, double *out);
int core_oracle_round(uint64_t seed, uint64_t round, uint64_t d, uint32_t m, uint32_t n, const void *G,
                      int dtype, uint64_t ld, const uint32_t *all_j, double *P, double *pbar, double *gtilde);

static int run_case(uint64_t d, uint32_t m, uint32_t n, int dtype, uint64_t ld)
{
    const size_t esz = dtype == 0 ? 8 : dtype == 1 ? 4 : 2;
    unsigned char *G = malloc((size_t)n * ld * esz);       /* exactly sized: overruns are caught */
    uint32_t *jidx = malloc(sizeof(uint32_t) * m);
    double *P = malloc(sizeof(double) * n * m), *pbar = malloc(sizeof(double) * m);
    double *gt = malloc(sizeof(double) * d);
    if (!G || !jidx || !P || !pbar || !gt) return 1;
    for (size_t t = 0; t < (size_t)n * ld; ++t) {
        const double v = sin(0.37 * (double)t) + 0.01 * (double)(t % 7);
        if (dtype == 0) ((double *)G)[t] = v;
        else if (dtype == 1) ((float *)G)[t] = (float)v;
        else { union { float f; uint32_t u; } c; c.f = (float)v; ((uint16_t *)G)[t] = (uint16_t)(c.u >> 16); }
    }
    for (uint32_t j = 0; j < m; ++j) jidx[j] = j;
    int rc = core_oracle_round(0xFFFFFFFF12345678ull, 1ull << 40, d, m, n, G, dtype, ld, jidx, P, pbar, gt);
    if (rc == 0) rc = core_oracle_compress(3, 4, d, n, G, dtype, ld, jidx, m, P);
    if (rc == 0) rc = core_oracle_client_mean(P, n, m, pbar);
    if (rc == 0 && d > 2) rc = core_oracle_reconstruct(3, 4, m, pbar, 1.0 / m, 1, d - 2, gt);
    for (uint64_t i = 0; rc == 0 && i + 2 < d; ++i) if (!isfinite(gt[i])) rc = 2;
    free(G); free(jidx); free(P); free(pbar); free(gt);
    return rc;
}

int main(void)
{
    const uint32_t ctr[4] = {0xffffffffu, 0xffffffffu, 0xffffffffu, 0xffffffffu}, key[2] = {0xffffffffu, 0xffffffffu};
    uint32_t w[4];
    core_oracle_philox4x32_10(ctr, key, w);
    if (w[0] != 0x408f276du) { fprintf(stderr, "philox known answer\n"); return 1; }
    double z[4];
    core_oracle_xi_block(~0ull, ~0ull, 0xffffffffu, 0xffffffffull, z);
    double buf[9];
    core_oracle_xi_fill(1, 2, 3, (1ull << 34) - 9, 9, buf);
    const uint64_t ds[] = {1, 2, 3, 4, 5, 7, 8, 9, 17};
    for (size_t a = 0; a < sizeof ds / sizeof ds[0]; ++a)
        for (uint32_t m = 1; m <= 3; ++m)
            for (uint32_t n = 1; n <= 3; ++n)
                for (int dtype = 0; dtype < 3; ++dtype) {
                    if (run_case(ds[a], m, n, dtype, ds[a])) { fprintf(stderr, "case failed\n"); return 1; }
                    if (run_case(ds[a], m, n, dtype, ds[a] + 3)) { fprintf(stderr, "padded case failed\n"); return 1; }
                }
    /* bad arguments are refused, not dereferenced */
    if (core_oracle_compress(1, 0, 4, 1, NULL, 1, 4, NULL, 0, NULL) == 0) return 1;
    if (core_oracle_reconstruct(1, 0, 0, NULL, 1.0, 0, 4, NULL) == 0) return 1;
    puts("oracle sanitizer run ok");
    return 0;
}
