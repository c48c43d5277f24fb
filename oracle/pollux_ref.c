/*
 * CPU checker ("oracle") for the PolluxSched search hot path -- see pollux_ref.h.
 * TEST INFRASTRUCTURE ONLY; shares no code with the GPU library.
 *
 * Plain fp64, one grid point at a time, in the order the paper writes the
 * formulas.  Compile with -ffp-contract=off so that no multiply-add is fused.
 * The only parallelism is an OpenMP loop over candidates.
 */
#include "pollux_ref.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* threads the candidate loop will use */
int pollux_ref_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ model */

/* Sec. 3.1, Eq. 6: EFFICIENCY_t(M) = (phi_t + M0) / (phi_t + M). */
double pollux_ref_efficiency(double phi, double M0, double M)
{
    return (phi + M0) / (phi + M);
}

/* Sec. 3.2, Eq. 8: T_grad(m) = alpha_grad + beta_grad * m. */
double pollux_ref_tgrad(double alpha_g, double beta_g, double m)
{
    return alpha_g + beta_g * m;
}

/* Sec. 3.2, Eq. 9: no synchronisation for one GPU; the "local" pair when all
 * K >= 2 replicas sit on one node; the "node" pair otherwise. */
double pollux_ref_tsync(const pollux_ref_job *job, int K, int nodes)
{
    if (K <= 1) return 0.0;
    if (nodes == 1) return job->alpha_sl + job->beta_sl * (double)(K - 2);
    return job->alpha_sn + job->beta_sn * (double)(K - 2);
}

/* Sec. 3.2, Eq. 10 (overlap of compute and synchronisation) inside Eq. 11
 * (s accumulation passes followed by one synchronised pass).  gamma = 1 is the
 * plain sum and T_sync = 0 leaves T_grad; both are taken exactly. */
double pollux_ref_titer(double t_grad, double t_sync, double gamma, int s)
{
    double last;
    if (t_sync == 0.0) last = t_grad;
    else if (gamma == 1.0) last = t_grad + t_sync;
    else last = pow(pow(t_grad, gamma) + pow(t_sync, gamma), 1.0 / gamma);
    return (double)s * t_grad + last;
}

/* Sec. 3, Eq. 4: GOODPUT = THROUGHPUT (Eq. 7: M / T_iter) x EFFICIENCY (Eq. 6),
 * with M = SUM(a) * m * (s + 1).  Only M0 <= M <= M_max is considered
 * (Sec. 3: batch sizes below the initial one are never used; Sec. 3.1: the
 * application's upper batch-size limit). */
double pollux_ref_goodput(const pollux_ref_job *job, int K, int nodes, int m, int s, int *feasible)
{
    if (feasible) *feasible = 0;
    if (K <= 0) return 0.0;
    double M = (double)K * (double)m * (double)(s + 1);
    if (M < job->M0 || M > job->Mmax) return 0.0;
    if (feasible) *feasible = 1;
    double t_grad = pollux_ref_tgrad(job->alpha_g, job->beta_g, (double)m);
    double t_sync = pollux_ref_tsync(job, K, nodes);
    double t_iter = pollux_ref_titer(t_grad, t_sync, job->gamma, s);
    double throughput = M / t_iter;
    double efficiency = pollux_ref_efficiency(job->phi, job->M0, M);
    return throughput * efficiency;
}

/* Sec. 4.1, Eq. 13: (m*, s*) = argmax over the grid; first strictly greater
 * value wins, i.e. ties go to the lowest flat index i_m * Gs + i_s. */
double pollux_ref_best_goodput(const pollux_ref_job *job, const int32_t *m_grid, int Gm, int Gs,
                               int K, int nodes, int *im, int *is)
{
    double best = 0.0;
    int bi = -1, bs = -1;
    for (int i = 0; i < Gm; ++i) {
        for (int s = 0; s < Gs; ++s) {
            int ok;
            double g = pollux_ref_goodput(job, K, nodes, m_grid[i], s, &ok);
            if (ok && g > best) { best = g; bi = i; bs = s; }
        }
    }
    if (im) *im = bi;
    if (is) *is = bs;
    return best;
}

/* Sec. 4.3: sample total batch sizes, derive (m, s) from the memory bound, keep the best.
 * The text's "m = ceil(M / s)" is read as m = ceil(M / (K (s+1))), consistent with
 * M = SUM(a) * m * (s+1) of Sec. 3. */
double pollux_ref_best_goodput_sampled(const pollux_ref_job *job, const int32_t *M_list, int count, int s_max,
                                       int K, int nodes, int *m_out, int *s_out)
{
    double best = 0.0;
    int bm = -1, bs = -1;
    if (K > 0 && job->m_mem >= 1.0) {
        for (int i = 0; i < count; ++i) {
            long long M = M_list[i];
            if (M <= 0) continue;
            long long per_step = (long long)K * (long long)job->m_mem;          /* examples one pass can hold */
            long long s = (M + per_step - 1) / per_step - 1;                     /* smallest s that fits */
            if (s > s_max) continue;
            long long m = (M + (long long)K * (s + 1) - 1) / ((long long)K * (s + 1));
            if (m > 2147483647LL) continue;
            int ok;
            double g = pollux_ref_goodput(job, K, nodes, (int)m, (int)s, &ok);
            if (ok && g > best) { best = g; bm = (int)m; bs = (int)s; }
        }
    }
    if (m_out) *m_out = bm;
    if (s_out) *s_out = bs;
    return best;
}

double pollux_ref_argmax_gap(const pollux_ref_job *job, const int32_t *m_grid, int Gm, int Gs,
                             int K, int nodes)
{
    if (K <= 0) return 1.0;
    long double best = 0.0L, second = 0.0L;
    long double ts = (long double)pollux_ref_tsync(job, K, nodes);
    for (int i = 0; i < Gm; ++i) {
        long double m = (long double)m_grid[i];
        long double tg = (long double)job->alpha_g + (long double)job->beta_g * m;
        long double last;
        if (ts == 0.0L) last = tg;
        else if (job->gamma == 1.0) last = tg + ts;
        else last = powl(powl(tg, (long double)job->gamma) + powl(ts, (long double)job->gamma),
                         1.0L / (long double)job->gamma);
        for (int s = 0; s < Gs; ++s) {
            long double M = (long double)K * m * (long double)(s + 1);
            if (M < (long double)job->M0 || M > (long double)job->Mmax) continue;
            long double g = (M / ((long double)s * tg + last)) *
                            (((long double)job->phi + (long double)job->M0) / ((long double)job->phi + M));
            if (g > best) { second = best; best = g; }
            else if (g < best && g > second) second = g;
        }
    }
    if (best <= 0.0L) return 1.0;
    return (double)((best - second) / best);
}

/* Sec. 4.2: REALLOC_FACTOR_j(delta) = (T_j - R_j * delta) / (T_j + delta). */
double pollux_ref_realloc_factor(double age_T, double restarts_R, double delta)
{
    return (age_T - restarts_R * delta) / (age_T + delta);
}

/* Sec. 4.2, Eq. 14 with job weights (all ones gives the paper's form):
 * ((sum_j w_j S_j^p) / (sum_j w_j))^(1/p), summed in ascending j; p = 0 is the
 * weighted geometric mean, its limit. */
double pollux_ref_pmean(const double *speedup, const double *weight, int J, double p)
{
    double acc = 0.0, wsum = 0.0;
    for (int j = 0; j < J; ++j) {
        double w = weight ? weight[j] : 1.0;
        wsum += w;
        if (p == 0.0) acc += w * log(speedup[j]);
        else acc += w * pow(speedup[j], p);
    }
    if (p == 0.0) return exp(acc / wsum);
    return pow(acc / wsum, 1.0 / p);
}

/* ---------------------------------------------------------------- fitness */

static void load_job(const double *jp, int J, int j, pollux_ref_job *job)
{
    job->alpha_g = jp[(size_t)PXR_ALPHA_G * J + j];
    job->beta_g = jp[(size_t)PXR_BETA_G * J + j];
    job->alpha_sl = jp[(size_t)PXR_ALPHA_SL * J + j];
    job->beta_sl = jp[(size_t)PXR_BETA_SL * J + j];
    job->alpha_sn = jp[(size_t)PXR_ALPHA_SN * J + j];
    job->beta_sn = jp[(size_t)PXR_BETA_SN * J + j];
    job->gamma = jp[(size_t)PXR_GAMMA * J + j];
    job->phi = jp[(size_t)PXR_PHI * J + j];
    job->M0 = jp[(size_t)PXR_M0 * J + j];
    job->Mmax = jp[(size_t)PXR_MMAX * J + j];
    job->m_mem = jp[(size_t)PXR_M_MEM * J + j];
}

static int job_is_bad(const pollux_ref_job *job, double weight)
{
    return !(job->gamma >= 1.0 && job->gamma <= 10.0) || !(job->alpha_g >= 0.0) || !(job->beta_g >= 0.0) ||
           !(job->alpha_sl >= 0.0) || !(job->beta_sl >= 0.0) || !(job->alpha_sn >= 0.0) ||
           !(job->beta_sn >= 0.0) || !(job->phi > 0.0) || !(job->M0 >= 1.0) || !(job->Mmax >= job->M0) ||
           !(weight >= 0.0) || !(job->Mmax <= 4503599627370496.0) || !(job->alpha_g + job->beta_g > 0.0);
}

int pollux_fitness_ref(const pollux_ref_dims *d, const int32_t *population, const double *job_params,
                       const int32_t *m_grid, const int32_t *fair_share, const int32_t *current_alloc,
                       const int32_t *node_capacity, double p, double delta, double *fitness,
                       int32_t *best_m, int32_t *best_s, double *best_goodput, double *speedup,
                       int32_t *violations, int32_t *status)
{
    if (!d || !population || !job_params || !m_grid || !fair_share || !current_alloc || !node_capacity ||
        !fitness || !best_m || !best_s)
        return -1;
    const int P = d->P, J = d->J, N = d->N, Gm = d->Gm, Gs = d->Gs;
    if (P <= 0 || J <= 0 || N <= 0 || Gm <= 0 || Gs <= 0 || !isfinite(p) || !isfinite(delta) || delta < 0.0)
        return -1;
    const int use_penalty = !(d->flags & 1), use_check = !(d->flags & 2), sampled = (d->flags & 16) != 0;
    int st = 0;

    /* per job: fair-share denominator of Eq. 15, restart factor, "has a current allocation" */
    double *denom = (double *)malloc(sizeof(double) * (size_t)J);
    double *factor = (double *)malloc(sizeof(double) * (size_t)J);
    int *running = (int *)malloc(sizeof(int) * (size_t)J);
    if (!denom || !factor || !running) { free(denom); free(factor); free(running); return -2; }
    for (int j = 0; j < J; ++j) {
        pollux_ref_job job;
        load_job(job_params, J, j, &job);
        double w = job_params[(size_t)PXR_WEIGHT * J + j];
        if (job_is_bad(&job, w) || (sampled && !(job.m_mem >= 1.0 && job.m_mem <= 2147483647.0))) st |= PXR_ST_BAD_PARAM;
        denom[j] = sampled
                       ? pollux_ref_best_goodput_sampled(&job, m_grid + (size_t)j * Gm, Gm, Gs - 1, fair_share[2 * j],
                                                         fair_share[2 * j + 1], NULL, NULL)
                       : pollux_ref_best_goodput(&job, m_grid + (size_t)j * Gm, Gm, Gs, fair_share[2 * j],
                                                 fair_share[2 * j + 1], NULL, NULL);
        if (!(denom[j] > 0.0)) st |= PXR_ST_ZERO_FAIR;
        double T = job_params[(size_t)PXR_AGE_T * J + j], R = job_params[(size_t)PXR_RESTARTS_R * J + j];
        factor[j] = pollux_ref_realloc_factor(T, R, delta);
        if (use_penalty && !(T - R * delta > 0.0)) st |= PXR_ST_BAD_RESTART;
        long csum = 0;
        for (int n = 0; n < N; ++n) {
            csum += current_alloc[(size_t)j * N + n];
            if (current_alloc[(size_t)j * N + n] < 0) st |= PXR_ST_NEG_ALLOC;
        }
        running[j] = csum > 0;
    }

    #pragma omp parallel for schedule(dynamic, 1) reduction(| : st)
    for (int c = 0; c < P; ++c) {
        const int32_t *A = population + (size_t)c * J * N;
        double *S = (double *)malloc(sizeof(double) * (size_t)J);
        int *nodes_of = (int *)malloc(sizeof(int) * (size_t)J);
        for (int j = 0; j < J; ++j) {
            const int32_t *row = A + (size_t)j * N;
            long K = 0;
            int nodes = 0, changed = 0;
            for (int n = 0; n < N; ++n) {
                K += row[n];
                nodes += row[n] > 0;
                changed |= row[n] != current_alloc[(size_t)j * N + n];
                if (row[n] < 0) st |= PXR_ST_NEG_ALLOC;
            }
            nodes_of[j] = nodes;
            pollux_ref_job job;
            load_job(job_params, J, j, &job);
            int im = -1, is = -1, m_star = -1;
            double g = 0.0;
            if (K > 0 && sampled) {
                g = pollux_ref_best_goodput_sampled(&job, m_grid + (size_t)j * Gm, Gm, Gs - 1, (int)K, nodes, &m_star, &is);
            } else if (K > 0) {
                g = pollux_ref_best_goodput(&job, m_grid + (size_t)j * Gm, Gm, Gs, (int)K, nodes, &im, &is);
                m_star = im >= 0 ? m_grid[(size_t)j * Gm + im] : -1;
            }
            size_t o = (size_t)c * J + j;
            best_m[o] = m_star;
            best_s[o] = is;
            if (best_goodput) best_goodput[o] = g;
            /* Eq. 15, then the re-allocation penalty for a job whose row differs
             * from its current one (a job with no current GPUs has nothing to restart) */
            double s_j = denom[j] > 0.0 ? g / denom[j] : 0.0;
            if (use_penalty && changed && running[j]) s_j = s_j * factor[j];
            S[j] = s_j;
            if (speedup) speedup[o] = s_j;
        }
        double f = pollux_ref_pmean(S, job_params + (size_t)PXR_WEIGHT * J, J, p);
        /* interference rule (at most one multi-node job per node) and node capacity */
        long V = 0;
        for (int n = 0; n < N; ++n) {
            long total = 0;
            int distributed = 0;
            for (int j = 0; j < J; ++j) {
                int32_t a = A[(size_t)j * N + n];
                total += a;
                if (a > 0 && nodes_of[j] >= 2) distributed++;
            }
            if (distributed > 1) V += distributed - 1;
            if (total > node_capacity[n]) V += total - node_capacity[n];
        }
        if (violations) violations[c] = (int32_t)V;
        fitness[c] = (use_check && V > 0) ? -(double)V : f;
        free(S);
        free(nodes_of);
    }
    if (status) *status = st;
    free(denom); free(factor); free(running);
    return 0;
}

/* ----------------------------------------------------------------- Philox */

/* Philox4x32 with 10 rounds: each round multiplies counter words 0 and 2 by
 * two fixed odd constants, keeps the low halves, and mixes the high halves
 * with the other two words and the key; the key is advanced by a Weyl
 * sequence between rounds. */
void pollux_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }
        uint64_t p0 = (uint64_t)0xD2511F53u * c0;
        uint64_t p1 = (uint64_t)0xCD9E8D57u * c2;
        uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)p1;
        uint32_t n2 = (uint32_t)(p0 >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)p0;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* --------------------------------------------------------------- GA step */

enum { TAG_PARENT = 0, TAG_CROSS = 1, TAG_MUT_DECIDE = 2, TAG_MUT_ARGS = 3, TAG_REPAIR = 4 };

static void draw(const uint32_t key[2], uint32_t generation, uint32_t child, uint32_t item, uint32_t tag,
                 uint32_t out[4])
{
    uint32_t ctr[4] = { generation, child, item, tag };
    pollux_ref_philox4x32_10(ctr, key, out);
}

static uint32_t below(uint32_t r, uint32_t n) { return (uint32_t)(((uint64_t)r * (uint64_t)n) >> 32); }

typedef struct { double f; int32_t idx; } ranked;

static int cmp_ranked(const void *a, const void *b)
{
    const ranked *x = (const ranked *)a, *y = (const ranked *)b;
    if (x->f > y->f) return -1;
    if (x->f < y->f) return 1;
    return x->idx < y->idx ? -1 : (x->idx > y->idx ? 1 : 0);
}

void pollux_ref_rank(const double *fitness, int P, int32_t *order)
{
    ranked *r = (ranked *)malloc(sizeof(ranked) * (size_t)P);
    for (int c = 0; c < P; ++c) {
        r[c].f = fitness[c] == fitness[c] ? fitness[c] : -INFINITY;
        r[c].idx = c;
    }
    qsort(r, (size_t)P, sizeof(ranked), cmp_ranked);
    for (int c = 0; c < P; ++c) order[c] = r[c].idx;
    free(r);
}

/* Make a matrix satisfy node capacity, then the one-multi-node-job-per-node
 * rule (Sec. 4.2 "Interference avoidance", Sec. 4.3).  Only removals. */
void pollux_ref_repair(int32_t *A, int J, int N, const int32_t *cap, const uint32_t key[2],
                       uint32_t generation, uint32_t child)
{
    /* capacity: node by node, take GPUs away walking the jobs cyclically from a drawn start */
    for (int n = 0; n < N; ++n) {
        long total = 0;
        for (int j = 0; j < J; ++j) total += A[(size_t)j * N + n];
        long excess = total - cap[n];
        if (excess <= 0) continue;
        uint32_t r[4];
        draw(key, generation, child, (uint32_t)n, TAG_REPAIR, r);
        int j0 = (int)below(r[0], (uint32_t)J);
        for (int t = 0; t < J && excess > 0; ++t) {
            int j = (j0 + t) % J;
            long have = A[(size_t)j * N + n];
            if (have <= 0) continue;
            long take = have < excess ? have : excess;
            A[(size_t)j * N + n] = (int32_t)(have - take);
            excess -= take;
        }
    }
    /* interference: nodes in ascending order; among the multi-node jobs present on a
     * node keep the one holding most GPUs there (lowest job index on a tie) */
    int *nodes_of = (int *)malloc(sizeof(int) * (size_t)J);
    for (int j = 0; j < J; ++j) {
        int c = 0;
        for (int n = 0; n < N; ++n) c += A[(size_t)j * N + n] > 0;
        nodes_of[j] = c;
    }
    for (int n = 0; n < N; ++n) {
        int keep = -1, count = 0;
        int32_t most = 0;
        for (int j = 0; j < J; ++j) {
            int32_t a = A[(size_t)j * N + n];
            if (a > 0 && nodes_of[j] >= 2) {
                count++;
                if (a > most) { most = a; keep = j; }
            }
        }
        if (count <= 1) continue;
        for (int j = 0; j < J; ++j) {
            if (j == keep) continue;
            if (A[(size_t)j * N + n] > 0 && nodes_of[j] >= 2) {
                A[(size_t)j * N + n] = 0;
                nodes_of[j] -= 1;
            }
        }
    }
    free(nodes_of);
}

/*
 * One generation of the population search (Sec. 4.3: perturb and combine
 * candidates, then modify them to satisfy the constraints).  The operators are
 * this project's own: the best elite_k candidates survive unchanged; every
 * other child takes each job's row from one of two drawn survivors, may grow or
 * shrink a row by one GPU on a node it occupies or re-pack it, and is repaired.
 */
/* Sec. 4.1 limits the GPUs a job may be given to twice the most it has ever held.  In the
 * search this is a repair on the row: walking the nodes in ascending order, the job keeps its
 * GPUs until `cap` of them are kept; what lies beyond is given back. */
void pollux_ref_cap_row(int32_t *row, int N, int32_t cap)
{
    long kept = 0, limit = cap > 0 ? cap : 0;
    for (int n = 0; n < N; ++n) {
        if (row[n] <= 0) continue;
        long room = limit - kept;
        if (row[n] > room) row[n] = (int32_t)room;
        kept += row[n];
    }
}

int pollux_ga_step_ref(const pollux_ref_dims *d, const int32_t *parents, const double *fitness,
                       const int32_t *cap, const pollux_ref_ga_params *ga, int32_t *children)
{
    if (!d || !parents || !fitness || !cap || !ga || !children) return -1;
    const int P = d->P, J = d->J, N = d->N;
    if (P <= 0 || J <= 0 || N <= 0 || ga->elite_k < 1 || ga->elite_k > (uint32_t)P) return -1;
    const uint32_t key[2] = { (uint32_t)(ga->seed & 0xFFFFFFFFu), (uint32_t)(ga->seed >> 32) };
    int32_t *order = (int32_t *)malloc(sizeof(int32_t) * (size_t)P);
    if (!order) return -2;
    pollux_ref_rank(fitness, P, order);
    const size_t JN = (size_t)J * N;
    /* in place (flags bit 0): the new generation is formed in a scratch copy exactly as below and
     * child c is then stored in the slot of the candidate of rank c, so survivors do not move */
    const int in_place = (ga->flags & 1u) != 0;
    int32_t *out = children;
    if (in_place) {
        out = (int32_t *)malloc(sizeof(int32_t) * JN * (size_t)P);
        if (!out) { free(order); return -2; }
    }

    #pragma omp parallel for schedule(dynamic, 1)
    for (int c = 0; c < P; ++c) {
        int32_t *child = out + (size_t)c * JN;
        if ((uint32_t)c < ga->elite_k) {
            memcpy(child, parents + (size_t)order[c] * JN, sizeof(int32_t) * JN);
            continue;
        }
        uint32_t r[4];
        draw(key, ga->generation, (uint32_t)c, 0u, TAG_PARENT, r);
        const int32_t *pa = parents + (size_t)order[below(r[0], ga->elite_k)] * JN;
        /* half of the children have a single parent (mutation only) */
        const int32_t *pb = (r[2] & 1u) ? pa : parents + (size_t)order[below(r[1], ga->elite_k)] * JN;
        for (int j = 0; j < J; ++j) {
            int32_t *row = child + (size_t)j * N;
            draw(key, ga->generation, (uint32_t)c, (uint32_t)j, TAG_CROSS, r);
            memcpy(row, ((r[0] & 1u) ? pb : pa) + (size_t)j * N, sizeof(int32_t) * (size_t)N);
            draw(key, ga->generation, (uint32_t)c, (uint32_t)j, TAG_MUT_DECIDE, r);
            if (r[0] < ga->mut_threshold) {
                draw(key, ga->generation, (uint32_t)c, (uint32_t)j, TAG_MUT_ARGS, r);
                uint32_t move = r[0] % 3u;
                int occupied = 0;
                for (int k = 0; k < N; ++k) occupied += row[k] > 0;
                if (move == 2u) {
                    /* re-pack: the whole row goes to one drawn node, as far as its capacity allows */
                    int n = (int)below(r[1], (uint32_t)N);
                    long K = 0;
                    for (int k = 0; k < N; ++k) { K += row[k]; row[k] = 0; }
                    if (K < 0) K = 0;
                    row[n] = (int32_t)(K < cap[n] ? K : cap[n]);
                } else if (occupied > 0) {
                    /* grow / shrink by one GPU on one of the nodes the job already occupies */
                    int pick = (int)below(r[1], (uint32_t)occupied), n = -1;
                    for (int k = 0; k < N; ++k) {
                        if (row[k] > 0 && pick-- == 0) { n = k; break; }
                    }
                    row[n] += (move == 0u) ? 1 : -1;
                } else if (move == 0u) {
                    /* a job without GPUs starts on a drawn node */
                    row[below(r[1], (uint32_t)N)] += 1;
                }
            }
            if (ga->job_gpu_cap) pollux_ref_cap_row(row, N, ga->job_gpu_cap[j]);
        }
        pollux_ref_repair(child, J, N, cap, key, ga->generation, (uint32_t)c);
    }
    if (in_place) {
        for (int c = 0; c < P; ++c) memcpy(children + (size_t)order[c] * JN, out + (size_t)c * JN, sizeof(int32_t) * JN);
        free(out);
    }
    free(order);
    return 0;
}
