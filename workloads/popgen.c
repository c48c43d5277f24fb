/*
 * Seeded synthetic allocation matrices for scheduler-search experiments.
 *
 * This file only produces INPUTS: int32 allocation matrices A[J][N]
 * (GPUs of node n given to job j) that respect a per-node capacity and the
 * rule that two multi-node jobs never meet on one node.  It contains none of
 * the goodput / fitness / genetic-operator arithmetic; both the CPU checker
 * and the GPU library consume the bytes it writes.
 *
 * Every candidate is a pure function of (seed, candidate index), so any
 * subset of a large population can be regenerated on its own.
 *
 * Random numbers: splitmix64 (Steele, Lea, Flood 2014; Vigna's constants),
 * one stream per candidate.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct { uint64_t s; } rng_t;

static uint64_t rng_u64(rng_t *r)
{
    uint64_t z = (r->s += 0x9E3779B97F4A7C15ull);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
static double rng_unit(rng_t *r) { return (double)(rng_u64(r) >> 11) * (1.0 / 9007199254740992.0); }
static uint32_t rng_below(rng_t *r, uint32_t n) { return (uint32_t)(((rng_u64(r) >> 32) * (uint64_t)n) >> 32); }
static double rng_normal(rng_t *r)
{
    double u1 = rng_unit(r), u2 = rng_unit(r);
    if (u1 < 1e-300) u1 = 1e-300;
    return sqrt(-2.0 * log(u1)) * cos(6.283185307179586 * u2);
}

static void rng_seed(rng_t *r, uint64_t seed, uint64_t index)
{
    r->s = seed ^ (0xD1B54A32D192ED03ull * (index + 1));
    (void)rng_u64(r);
    (void)rng_u64(r);
}

/* Packed fair-share matrix: job j gets kf GPUs, first fit, never straddling
 * a node boundary when kf <= cap. */
static void fill_fair(int32_t *A, int J, int N, int cap, int kf)
{
    memset(A, 0, sizeof(int32_t) * (size_t)J * N);
    int node = 0, used = 0;
    for (int j = 0; j < J; ++j) {
        int want = kf;
        if (want <= cap && used + want > cap) { node++; used = 0; }
        while (want > 0 && node < N) {
            int take = cap - used < want ? cap - used : want;
            A[(size_t)j * N + node] += take;
            used += take; want -= take;
            if (used == cap) { node++; used = 0; }
        }
    }
}

/*
 * One random candidate.  Jobs are visited in a seeded random order; each
 * draws a GPU count around the fair share (log-normal, sigma 0.7) and is
 * either packed into as few nodes as possible from a random start node
 * (probability 0.7) or scattered one GPU at a time.  `owner[n]` records the
 * multi-node job that holds node n, so the no-sharing rule holds by
 * construction.  When `allow_zero` is set each job is left without GPUs with
 * probability 2 % (a pending job).
 */
static void fill_random(int32_t *A, int J, int N, int cap, int kf, rng_t *r, int allow_zero,
                        int32_t *freecap, int32_t *owner, int32_t *order, int32_t *mine)
{
    memset(A, 0, sizeof(int32_t) * (size_t)J * N);
    for (int n = 0; n < N; ++n) { freecap[n] = cap; owner[n] = -1; }
    for (int j = 0; j < J; ++j) order[j] = j;
    for (int j = J - 1; j > 0; --j) {
        int k = (int)rng_below(r, (uint32_t)j + 1);
        int32_t t = order[j]; order[j] = order[k]; order[k] = t;
    }
    long free_total = (long)N * cap;
    for (int t = 0; t < J; ++t) {
        int j = order[t];
        int32_t *row = A + (size_t)j * N;
        int remaining_jobs = J - 1 - t;
        double z = rng_normal(r);
        double pick = rng_unit(r), zero = rng_unit(r);
        uint32_t start = rng_below(r, (uint32_t)N);
        long K = lround((double)kf * exp(0.7 * z));
        if (K < 1) K = 1;
        if (K > 4L * cap) K = 4L * cap;
        long budget = free_total - remaining_jobs;       /* leave one GPU for every later job */
        if (K > budget) K = budget;
        if (allow_zero && zero < 0.02) K = 0;
        if (K <= 0) continue;
        int nmine = 0;
        if (pick < 0.7) {
            /* packed: a single node if one has room, else consecutive free nodes */
            int placed = 0;
            for (int d = 0; d < N && !placed; ++d) {
                int n = (int)((start + (uint32_t)d) % (uint32_t)N);
                if (freecap[n] >= K) { row[n] = (int32_t)K; freecap[n] -= (int32_t)K; free_total -= K; placed = 1; }
            }
            if (placed) continue;
            long want = K;
            for (int d = 0; d < N && want > 0; ++d) {
                int n = (int)((start + (uint32_t)d) % (uint32_t)N);
                if (freecap[n] <= 0 || owner[n] >= 0) continue;
                int take = freecap[n] < want ? freecap[n] : (int)want;
                row[n] += take; freecap[n] -= take; free_total -= take; want -= take;
                mine[nmine++] = n;
            }
        } else {
            /* scattered: one GPU at a time on random nodes not held by another multi-node job */
            for (long g = 0; g < K; ++g) {
                int n = -1;
                for (int attempt = 0; attempt < 8 && n < 0; ++attempt) {
                    int c = (int)rng_below(r, (uint32_t)N);
                    if (freecap[c] > 0 && (owner[c] < 0 || owner[c] == j)) n = c;
                }
                if (n < 0) {
                    for (int d = 0; d < N && n < 0; ++d) {
                        int c = (int)((start + (uint32_t)d) % (uint32_t)N);
                        if (freecap[c] > 0 && (owner[c] < 0 || owner[c] == j)) n = c;
                    }
                }
                if (n < 0) break;
                if (row[n] == 0) { mine[nmine++] = n; owner[n] = j; }
                row[n] += 1; freecap[n] -= 1; free_total -= 1;
            }
        }
        if (nmine >= 2) { for (int k = 0; k < nmine; ++k) owner[mine[k]] = j; }
        else            { for (int k = 0; k < nmine; ++k) if (owner[mine[k]] == j) owner[mine[k]] = -1; }
        if (nmine == 0) {
            /* nothing placed under the sharing rule: fall back to one GPU anywhere */
            for (int d = 0; d < N; ++d) {
                int n = (int)((start + (uint32_t)d) % (uint32_t)N);
                if (freecap[n] > 0) { row[n] += 1; freecap[n] -= 1; free_total -= 1; break; }
            }
        }
    }
}

/* Deliberately break a candidate: overload one node and spread one job so
 * that constraint checks have something to find. */
static void spoil(int32_t *A, int J, int N, int cap, rng_t *r)
{
    int j = (int)rng_below(r, (uint32_t)J), n = (int)rng_below(r, (uint32_t)N);
    A[(size_t)j * N + n] += cap;
    int j2 = (int)rng_below(r, (uint32_t)J);
    for (int k = 0; k < 3; ++k) A[(size_t)j2 * N + rng_below(r, (uint32_t)N)] += 1;
}

/*
 * kind of candidate `idx`:
 *   idx == 0            packed fair share
 *   idx % 20 == 7       random, then spoiled (infeasible on purpose)
 *   idx % 10 == 3       random with pending (zero-GPU) jobs
 *   otherwise           random, every job holds at least one GPU
 * Candidate index P (one past the population) is used for the current
 * allocation; it follows the same rule.
 */
int popgen_candidates(uint64_t seed, int64_t first, int64_t count, int J, int N, int cap, int kf,
                      int32_t *out /* [count][J][N] */)
{
    if (J <= 0 || N <= 0 || cap <= 0 || kf <= 0 || count < 0 || !out) return -1;
    int err = 0;
    #pragma omp parallel
    {
        int32_t *freecap = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
        int32_t *owner = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
        int32_t *mine = (int32_t *)malloc(sizeof(int32_t) * (size_t)N);
        int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)J);
        if (!freecap || !owner || !mine || !order) {
            #pragma omp atomic write
            err = -2;
        } else {
            #pragma omp for schedule(dynamic, 4)
            for (int64_t c = 0; c < count; ++c) {
                int64_t idx = first + c;
                int32_t *A = out + (size_t)c * J * N;
                if (idx == 0) { fill_fair(A, J, N, cap, kf); continue; }
                rng_t r; rng_seed(&r, seed, (uint64_t)idx);
                fill_random(A, J, N, cap, kf, &r, idx % 10 == 3, freecap, owner, order, mine);
                if (idx % 20 == 7) spoil(A, J, N, cap, &r);
            }
        }
        free(freecap); free(owner); free(mine); free(order);
    }
    return err;
}
