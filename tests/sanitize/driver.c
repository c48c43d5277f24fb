/*
 * Runs the CPU checker and the input generator under the address and undefined-behaviour sanitizers
 * (test infrastructure; built and run by tests/test_oracle_sanitizers.py, never by the GPU library).
 *
 * For a few small cluster shapes, including ragged ones: draw a population with popgen_candidates,
 * draw job parameters from a small generator of its own, then alternate pollux_fitness_ref and
 * pollux_ga_step_ref (out of place and in place, with and without per-job GPU limits, plain and
 * sampling argmax) for a few generations.  Every buffer is exactly as large as the interface says, so
 * an access outside one is reported.  Prints one checksum line per shape; exit status 0 on success.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "../../oracle/pollux_ref.h"

int popgen_candidates(uint64_t seed, int64_t first, int64_t count, int J, int N, int cap, int kf, int32_t *out);

static uint64_t state = 0x2008122600000001ull;
static double unit(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(state >> 11) * (1.0 / 9007199254740992.0);
}
static double between(double lo, double hi) { return lo + (hi - lo) * unit(); }

static int run_shape(int P, int J, int N, int cap, int Gm, int Gs, int flags)
{
    const size_t JN = (size_t)J * N;
    int32_t *pop = malloc(sizeof(int32_t) * P * JN), *next = malloc(sizeof(int32_t) * P * JN);
    int32_t *cur = malloc(sizeof(int32_t) * JN), *capn = malloc(sizeof(int32_t) * N);
    int32_t *grid = malloc(sizeof(int32_t) * (size_t)J * Gm), *fair = malloc(sizeof(int32_t) * 2 * J);
    int32_t *limit = malloc(sizeof(int32_t) * J);
    double *jp = malloc(sizeof(double) * PXR_NPARAM * J), *fit = malloc(sizeof(double) * P);
    int32_t *bm = malloc(sizeof(int32_t) * (size_t)P * J), *bs = malloc(sizeof(int32_t) * (size_t)P * J);
    double *bg = malloc(sizeof(double) * (size_t)P * J), *sp = malloc(sizeof(double) * (size_t)P * J);
    int32_t *viol = malloc(sizeof(int32_t) * P);
    int kf = (N * cap) / J;
    if (kf < 1) kf = 1;
    if (popgen_candidates(0x5EED2008ull + (uint64_t)J, 0, P, J, N, cap, kf, pop) != 0) return 1;
    if (popgen_candidates(0x5EED2008ull + (uint64_t)J, P, 1, J, N, cap, kf, cur) != 0) return 1;
    for (int n = 0; n < N; ++n) capn[n] = cap;
    for (int j = 0; j < J; ++j) {
        double m_max = floor(between(64.0, 513.0)), M0 = 32.0 * (double)(1 << (int)(unit() * 4.0));
        jp[PXR_ALPHA_G * J + j] = between(0.01, 0.2);
        jp[PXR_BETA_G * J + j] = exp(between(log(1e-5), log(1e-3)));
        jp[PXR_ALPHA_SL * J + j] = between(0.005, 0.05);
        jp[PXR_BETA_SL * J + j] = between(0.001, 0.01);
        jp[PXR_ALPHA_SN * J + j] = between(0.02, 0.2);
        jp[PXR_BETA_SN * J + j] = between(0.005, 0.05);
        jp[PXR_GAMMA * J + j] = j % 5 == 0 ? 1.0 : between(1.0, 5.0);
        jp[PXR_PHI * J + j] = exp(between(log(1e2), log(1e5)));
        jp[PXR_M0 * J + j] = M0;
        jp[PXR_MMAX * J + j] = 32.0 * M0;
        jp[PXR_WEIGHT * J + j] = 1.0;
        jp[PXR_AGE_T * J + j] = between(120.0, 28800.0);
        jp[PXR_RESTARTS_R * J + j] = floor(unit() * jp[PXR_AGE_T * J + j] / 210.0);
        jp[PXR_M_MEM * J + j] = m_max;
        for (int i = 0; i < Gm; ++i) {
            double t = Gm > 1 ? (double)i / (Gm - 1) : 1.0;
            double v = (flags & 16) ? floor(M0 * pow(32.0, t) + 0.5) : floor(8.0 * pow(m_max / 8.0, t) + 0.5);
            grid[(size_t)j * Gm + i] = (int32_t)v;
        }
        fair[2 * j] = kf;
        fair[2 * j + 1] = (kf + cap - 1) / cap;
        limit[j] = (int32_t)(unit() * 6.0);
    }
    pollux_ref_dims d = { P, J, N, Gm, Gs, 0, flags };
    double sum = 0.0;
    long cells = 0;
    for (int gen = 0; gen < 4; ++gen) {
        int32_t st = 0;
        if (pollux_fitness_ref(&d, pop, jp, grid, fair, cur, capn, gen % 2 ? 0.5 : -1.0, 30.0, fit, bm, bs,
                               gen % 2 ? bg : NULL, gen % 2 ? NULL : sp, gen == 3 ? NULL : viol, gen == 2 ? NULL : &st) != 0)
            return 2;
        for (int c = 0; c < P; ++c) sum += isfinite(fit[c]) ? fit[c] : 0.0;
        pollux_ref_ga_params ga = { 0x20081226ull << 8, (uint32_t)gen, (uint32_t)(gen == 1 ? 1 : (P + 1) / 2),
                                    gen == 2 ? 0xFFFFFFFFu : 1u << 30, (uint32_t)(gen % 2), gen >= 2 ? limit : NULL };
        if (gen % 2) {
            if (pollux_ga_step_ref(&d, pop, fit, capn, &ga, pop) != 0) return 3;          /* in place */
        } else {
            if (pollux_ga_step_ref(&d, pop, fit, capn, &ga, next) != 0) return 3;
            memcpy(pop, next, sizeof(int32_t) * P * JN);
        }
        for (size_t e = 0; e < P * JN; ++e) cells += pop[e];
    }
    printf("P=%d J=%d N=%d cap=%d Gm=%d Gs=%d flags=%d fitness sum %.12g GPUs %ld\n", P, J, N, cap, Gm, Gs, flags, sum, cells);
    free(pop); free(next); free(cur); free(capn); free(grid); free(fair); free(limit); free(jp); free(fit);
    free(bm); free(bs); free(bg); free(sp); free(viol);
    return 0;
}

int main(void)
{
    static const int shapes[][7] = {
        /* P   J   N  cap  Gm  Gs flags */
        { 16,  8,  4,  4, 32,  8, 0 },
        { 24, 30, 16,  4, 64, 16, 0 },
        {  5,  7,  3,  4,  5,  3, 0 },
        {  3,  1,  1,  8,  1,  1, 0 },
        {  9, 13, 67,  2, 70,  5, 0 },
        {  6, 40,  9, 40, 33,  5, 0 },
        { 16,  8,  4,  4, 32,  8, 16 },
        {  9, 13, 67,  2, 70,  5, 16 },
        { 12, 11,  5,  4,  7,  4, 3 },
    };
    for (size_t k = 0; k < sizeof(shapes) / sizeof(shapes[0]); ++k) {
        const int *s = shapes[k];
        int rc = run_shape(s[0], s[1], s[2], s[3], s[4], s[5], s[6]);
        if (rc != 0) { fprintf(stderr, "shape %zu failed with %d\n", k, rc); return rc; }
    }
    return 0;
}
