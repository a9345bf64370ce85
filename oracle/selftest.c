/* Small driver for running the oracle under the host sanitizers (test infrastructure): one round of FO-SGD on a
 * few geometries, every array exactly sized, so that an out-of-bounds access or undefined operation in the
 * oracle aborts the run.  Prints a checksum; exit status 0 means the sanitizers saw nothing. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>

#include "fo_oracle.c"

static int run(uint64_t d, uint32_t M, uint32_t blk, uint32_t K, uint32_t eps_mode, uint32_t server_scale)
{
    orc_params p = { d, M, blk, K, ORC_DITHER_UNIFORM, ORC_SCALE_L2, eps_mode, 2.0, 2.0, 1.0, 77, server_scale };
    uint64_t b, nb, ntot;
    orc_geometry(&p, &b, &nb, &ntot);
    float **g = (float **)malloc(M * sizeof(float *));
    for (uint32_t m = 0; m < M; ++m) {
        g[m] = (float *)malloc(d * sizeof(float));
        for (uint64_t i = 0; i < d; ++i) g[m][i] = (float)sin(0.37 * (double)(i + 1) * (m + 1));
    }
    double *x = (double *)calloc(d, sizeof(double));
    uint64_t *bits_up = (uint64_t *)malloc((size_t)M * (ntot / 64) * sizeof(uint64_t));
    double *lam_up = (double *)malloc((size_t)M * nb * sizeof(double));
    double *gbar = (double *)malloc(ntot * sizeof(double));
    uint64_t *bits_down = (uint64_t *)malloc((ntot / 64) * sizeof(uint64_t));
    double *lam_s = (double *)malloc(nb * sizeof(double));
    double *gd = (double *)malloc(d * sizeof(double));
    for (uint64_t round = 0; round < 3; ++round)
        orc_round(&p, (const float *const *)g, x, 0.1, round, 2, bits_up, lam_up, gbar, bits_down, lam_s, gd);
    double cs = 0.0;
    for (uint64_t i = 0; i < d; ++i) cs += x[i] * (double)(i % 7 + 1);
    printf("d=%llu M=%u blk=%u K=%u eps=%u srv=%u n=%llu checksum %.12g\n", (unsigned long long)d, M, blk, K, eps_mode,
           server_scale, (unsigned long long)ntot, cs);
    for (uint32_t m = 0; m < M; ++m) free(g[m]);
    free(g); free(x); free(bits_up); free(lam_up); free(gbar); free(bits_down); free(lam_s); free(gd);
    return isfinite(cs) ? 0 : 1;
}

int main(void)
{
    int rc = 0;
    rc |= run(1, 1, 0, 1, 0, 0);
    rc |= run(100, 3, 0, 1, 0, 0);
    rc |= run(1000, 2, 6, 3, 1, 1);
    rc |= run(5000, 4, 8, 1, 2, 1);
    rc |= run(70000, 2, 0, 2, 0, 1);
    return rc;
}
