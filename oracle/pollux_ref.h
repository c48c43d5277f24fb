/*
 * CPU checker ("oracle") for the PolluxSched search hot path.
 *
 * TEST INFRASTRUCTURE ONLY.  This is a plain, slow, fp64 transcription of the
 * definitions in the Pollux paper (arXiv 2008.12260): the goodput model
 * (Sec. 3, Eq. 4; Sec. 3.1, Eq. 6; Sec. 3.2, Eq. 7-11), the per-job argmax
 * over (m, s) (Sec. 4.1, Eq. 13), SPEEDUP / FITNESS_p with the re-allocation
 * penalty and the interference rule (Sec. 4.2, Eq. 14-15), and one step of the
 * population search (Sec. 4.3).  It shares no code with the GPU library and
 * must never be linked or called by it.
 *
 * All pointers are HOST pointers.  Nothing is allocated that outlives a call.
 *
 * Parity status: every function below is pinned by the CPU test-suite to
 * closed forms, hand-derived values, brute force or invariants, EXCEPT the
 * choice of genetic operators in pollux_ga_step_ref: the paper only says that
 * candidates are perturbed, combined and then modified to satisfy the
 * constraints, so the operators are this project's own definition.  They are
 * pinned by their invariants only -- "parity unpinned" with respect to the
 * paper.
 */
#ifndef POLLUX_REF_H
#define POLLUX_REF_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct {
    int32_t P, J, N, Gm, Gs;
    int32_t precision; /* ignored: the oracle is always fp64 */
    int32_t flags;     /* bit0: no re-allocation penalty; bit1: no constraint check;
                          bit4 (16): Eq. 13 by sampling total batch sizes (Sec. 4.3) instead of the (m,s) grid */
} pollux_ref_dims;

/* rows of job_params[NPARAM][J] */
enum {
    PXR_ALPHA_G, PXR_BETA_G, PXR_ALPHA_SL, PXR_BETA_SL, PXR_ALPHA_SN, PXR_BETA_SN,
    PXR_GAMMA, PXR_PHI, PXR_M0, PXR_MMAX, PXR_WEIGHT, PXR_AGE_T, PXR_RESTARTS_R, PXR_M_MEM, PXR_NPARAM
};

/* data-dependent conditions, OR-ed into *status */
enum {
    PXR_ST_BAD_PARAM = 1,      /* gamma outside [1,10], negative alpha/beta/weight, phi<=0, M0<1, M_max<M0,
                                  M_max > 2^52 (M no longer exact in fp64), alpha_grad = beta_grad = 0 (T_grad = 0) */
    PXR_ST_ZERO_FAIR = 2,      /* fair-share goodput is zero: SPEEDUP set to 0 */
    PXR_ST_BAD_RESTART = 4,    /* T_j - R_j*delta <= 0 */
    PXR_ST_NEG_ALLOC = 8       /* a negative entry in an allocation matrix */
};

typedef struct {
    double alpha_g, beta_g, alpha_sl, beta_sl, alpha_sn, beta_sn, gamma, phi, M0, Mmax;
    double m_mem;      /* largest per-GPU batch size that fits GPU memory (sampling mode only) */
} pollux_ref_job;

/* --- pieces of the model, exposed so that each can be pinned on its own --- */
double pollux_ref_efficiency(double phi, double M0, double M);                 /* Eq. 6  */
double pollux_ref_tgrad(double alpha_g, double beta_g, double m);              /* Eq. 8  */
double pollux_ref_tsync(const pollux_ref_job *job, int K, int nodes);          /* Eq. 9  */
double pollux_ref_titer(double t_grad, double t_sync, double gamma, int s);    /* Eq. 10-11 */
/* Eq. 4 at one point; *feasible = 0 (and 0 returned) when M is outside [M0, M_max] or K<=0 */
double pollux_ref_goodput(const pollux_ref_job *job, int K, int nodes, int m, int s, int *feasible);
/* Eq. 13 over the grid m_grid[0..Gm) x s in 0..Gs-1; ties -> lowest i_m*Gs+i_s.
 * Returns the best goodput (0 when nothing is feasible; then *im = *is = -1). */
double pollux_ref_best_goodput(const pollux_ref_job *job, const int32_t *m_grid, int Gm, int Gs,
                               int K, int nodes, int *im, int *is);
/* Eq. 13 the way Sec. 4.3 describes it: for each candidate total batch size M_i the
 * smallest s whose per-GPU batch size m = ceil(M_i / (K (s+1))) fits GPU memory
 * (m <= m_mem, s <= s_max), then the best GOODPUT among those configurations; ties ->
 * lowest i.  *m and *s receive the chosen configuration (-1/-1 if none is feasible). */
double pollux_ref_best_goodput_sampled(const pollux_ref_job *job, const int32_t *M_list, int count, int s_max,
                                       int K, int nodes, int *m, int *s);
/* Same sweep in long double: relative gap between the best value and the best
 * strictly smaller value (1.0 when there is no runner-up).  Used to tell a
 * genuine mismatch from a tie below fp64 resolution. */
double pollux_ref_argmax_gap(const pollux_ref_job *job, const int32_t *m_grid, int Gm, int Gs,
                             int K, int nodes);
double pollux_ref_realloc_factor(double age_T, double restarts_R, double delta); /* Sec. 4.2 */
double pollux_ref_pmean(const double *speedup, const double *weight, int J, double p); /* Eq. 14 */

/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw, SC'11) */
void pollux_ref_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4]);

/* threads used by the loop over candidates */
int pollux_ref_threads(void);

/* --- whole calls --- */
int pollux_fitness_ref(const pollux_ref_dims *dims,
                       const int32_t *population,    /* [P,J,N] */
                       const double *job_params,     /* [PXR_NPARAM,J] */
                       const int32_t *m_grid,        /* [J,Gm] */
                       const int32_t *fair_share,    /* [J,2] (GPUs, nodes) */
                       const int32_t *current_alloc, /* [J,N] */
                       const int32_t *node_capacity, /* [N] */
                       double p, double delta,
                       double *fitness,              /* [P] out */
                       int32_t *best_m, int32_t *best_s, /* [P,J] out, -1/-1 when goodput is 0 */
                       double *best_goodput,         /* [P,J] out, may be NULL */
                       double *speedup,              /* [P,J] out, may be NULL (after penalty) */
                       int32_t *violations,          /* [P] out, may be NULL */
                       int32_t *status);             /* out, may be NULL */

typedef struct {
    uint64_t seed;
    uint32_t generation;
    uint32_t elite_k;
    uint32_t mut_threshold; /* floor(probability * 2^32) */
    uint32_t flags;
    const int32_t *job_gpu_cap; /* [J] or NULL: most GPUs job j may hold in a child (Sec. 4.1: twice its lifetime maximum) */
} pollux_ref_ga_params;

int pollux_ga_step_ref(const pollux_ref_dims *dims, const int32_t *parents, const double *fitness,
                       const int32_t *node_capacity, const pollux_ref_ga_params *ga,
                       int32_t *children /* [P,J,N], must not alias parents */);

/* the per-job GPU limit on one row, in place: GPUs are kept in ascending node order up to `cap` */
void pollux_ref_cap_row(int32_t *row, int N, int32_t cap);
/* repair alone (capacity, then interference) on one matrix A[J][N], in place */
void pollux_ref_repair(int32_t *A, int J, int N, const int32_t *node_capacity,
                       const uint32_t key[2], uint32_t generation, uint32_t child);
/* rank alone: order[0..P) by (fitness desc, index asc), NaN ranks last */
void pollux_ref_rank(const double *fitness, int P, int32_t *order);

#ifdef __cplusplus
}
#endif
#endif
