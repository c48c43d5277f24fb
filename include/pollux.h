/*
 * pollux.h -- C ABI of the MI355X (gfx950) library for the PolluxSched search
 * hot path (Pollux, arXiv 2008.12260, Sec. 4.2-4.3): batched fitness evaluation
 * of a population of allocation matrices, and one step of the population
 * search.
 *
 * Conventions
 *   - Every data pointer is a DEVICE pointer unless its comment says "host".
 *     All buffers are owned by the caller; inputs are never written.
 *   - Work is enqueued on the HIP stream passed as `hip_stream` (a hipStream_t
 *     cast to void*, NULL = the default stream).  No call synchronises the
 *     host except pollux_last_status.  Outputs are valid once the caller has
 *     synchronised the stream.
 *   - No call allocates or frees device memory; scratch space is the
 *     caller-provided `workspace` (size from pollux_workspace_size, 256-byte
 *     aligned).  Two calls that overlap in time must use different workspaces.
 *     pollux_fitness_static uses an array inside the library instead.
 *   - Return value: PX_OK (0) or a negative PX_E_* code.  Arguments that can be
 *     checked on the host are checked before anything is launched.  Conditions
 *     that depend on device data are OR-ed into a status word inside the
 *     workspace (PX_ST_* bits), read back with pollux_last_status.
 *   - Matrices are row-major with the last index contiguous.
 *   - The library keeps no state between calls that changes what a call computes or
 *     enqueues; calls from several threads or on several streams are independent as
 *     long as their workspaces differ (pollux_fitness_static: see there).
 */
#ifndef POLLUX_H
#define POLLUX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define POLLUX_VERSION 105

typedef struct {
    int32_t P;         /* candidates in the population                          */
    int32_t J;         /* jobs (running and pending), rows of an allocation matrix */
    int32_t N;         /* nodes, columns of an allocation matrix                */
    int32_t Gm;        /* points of the per-GPU batch-size grid of each job, at most 2^20 */
    int32_t Gs;        /* gradient-accumulation steps considered: s = 0..Gs-1, at most 2^14;
                          (Gm + 63) x (Gs rounded up to a multiple of 32) at most 2^28   */
    int32_t precision; /* 0 = fp64 arithmetic, 1 = fp32 arithmetic              */
    int32_t flags;     /* PX_FLAG_* */
} pollux_dims;

enum {
    PX_FLAG_NO_REALLOC_PENALTY = 1,   /* skip the re-allocation penalty of Sec. 4.2         */
    PX_FLAG_NO_CONSTRAINT_CHECK = 2,  /* fitness is Eq. 14 even for infeasible candidates  */
    PX_FLAG_MEMOISE = 4,              /* sweep the (m, s) grid once per (job, K, one node or several) instead of
                                         once per (candidate, job): the goodput model (Eq. 4, 9) sees a row only
                                         through those; identical results, the population pass becomes a gather */
    PX_FLAG_KEEP_JOB_TABLES = 8,      /* reuse what the previous pollux_fitness call on this workspace derived from
                                         the jobs alone (tables, fair-share goodput, restart factors, memoised
                                         sweeps): the caller guarantees that dims, job_params, m_grid, fair_share,
                                         current_alloc, delta and the other flags are unchanged since that call
                                         and that nothing but this library has written to the workspace,
                                         as in the generations of one scheduling interval.  The status word is
                                         then not cleared and keeps accumulating. */
    PX_FLAG_SAMPLE_M = 16,            /* the argmax of Eq. 13 by the sampling procedure of Sec. 4.3 instead of the
                                         dense grid: m_grid[j,*] then holds candidate TOTAL batch sizes M, and for
                                         each one s is the smallest count with which the per-GPU batch fits
                                         PX_M_MEM; see pollux_fitness.  fp64 only. */
    PX_FLAG_PAIR_RESULTS = 32         /* with PX_FLAG_MEMOISE: the call also leaves the goodput and the node count of
                                         every (candidate, job) pair in the workspace, which pollux_generation with
                                         PX_GA_INHERIT_ROWS reads (calls without PX_FLAG_MEMOISE leave them anyway;
                                         a memoised call on rows of 65 to 256 nodes otherwise keeps them on chip,
                                         and the 12 bytes per pair cost it about a twentieth of its time). */
};

/* Rows of job_params[PX_NPARAM][J] (structure of arrays, fp64).
 * The first seven are theta_sys of Sec. 4.1 (Eq. 12); PHI and M0 complete the
 * goodput-function triple (theta_sys, phi_t, M0) each job reports. */
enum {
    PX_ALPHA_G = 0,   /* alpha_grad  [s]           Eq. 8  */
    PX_BETA_G,        /* beta_grad   [s / example] Eq. 8  */
    PX_ALPHA_SL,      /* alpha_sync^local          Eq. 9  */
    PX_BETA_SL,       /* beta_sync^local           Eq. 9  */
    PX_ALPHA_SN,      /* alpha_sync^node           Eq. 9  */
    PX_BETA_SN,       /* beta_sync^node            Eq. 9  */
    PX_GAMMA,         /* overlap exponent, 1 <= gamma <= 10 (Eq. 10, Sec. 4.1) */
    PX_PHI,           /* pre-conditioned gradient noise scale phi_t > 0 (Eq. 5-6) */
    PX_M0,            /* initial batch size M0 >= 1 (Sec. 3)                     */
    PX_MMAX,          /* upper batch-size limit, M0 <= M_max <= 2^52 (Sec. 3.1)  */
    PX_WEIGHT,        /* weight of the job in the generalized mean, >= 0        */
    PX_AGE_T,         /* age T_j of the job [s] (Sec. 4.2, re-allocation penalty) */
    PX_RESTARTS_R,    /* re-allocations R_j so far                               */
    PX_M_MEM,         /* largest per-GPU batch size that fits GPU memory (Sec. 4.3), 1..2^31-1;
                         read only with PX_FLAG_SAMPLE_M                         */
    PX_NPARAM
};

enum {
    PX_OK = 0,
    PX_E_INVALID_ARG = -1,       /* null pointer, non-positive size, non-finite p or delta, delta < 0,
                                    unknown precision, elite_k outside 1..P, aliasing children/parents,
                                    a shape beyond a documented limit */
    PX_E_WORKSPACE = -2,         /* workspace null, misaligned or smaller than pollux_workspace_size */
    PX_E_UNSUPPORTED_ARCH = -3,  /* the current device is not gfx950 */
    PX_E_HIP = -4                /* a HIP runtime call failed (launch, attribute query, copy) */
};

/* bits of the status word */
enum {
    PX_ST_BAD_PARAM = 1,    /* a job parameter outside the domain documented at PX_* above,
                               or alpha_grad = beta_grad = 0; what is reported for such a job
                               (and the fitness of every candidate, which averages over it) is
                               then unspecified, the other jobs' results are unaffected */
    PX_ST_ZERO_FAIR = 2,    /* a job's fair-share goodput is 0: its SPEEDUP is set to 0 */
    PX_ST_BAD_RESTART = 4,  /* T_j - R_j * delta <= 0 for some job (penalty enabled) */
    PX_ST_NEG_ALLOC = 8     /* a negative entry in population or current_alloc */
};

/* Bytes of workspace needed by pollux_fitness and pollux_ga_step for `dims`
 * (one figure that covers both).  Host call, no device access. */
int pollux_workspace_size(const pollux_dims *dims, size_t *bytes /* host, out */);

/*
 * FITNESS_p of every candidate (Sec. 4.2, Eq. 14) with the per-job tuning it
 * needs (Sec. 4.1, Eq. 13).
 *
 * For candidate c and job j, with K = sum_n A[c,j,n] GPUs on
 * nodes = #{n : A[c,j,n] > 0} nodes, the goodput model (Eq. 4 = Eq. 7 x Eq. 6,
 * with Eq. 8-11) is evaluated at every point of the grid
 * m in m_grid[j,0..Gm), s in 0..Gs-1 with total batch size
 * M = K*m*(s+1) restricted to M0 <= M <= M_max, and the maximum is taken; ties
 * go to the lowest flat index i_m*Gs + s.  SPEEDUP_j (Eq. 15) divides by the
 * same maximum for the fair-share allocation (fair_share[j] = GPUs, nodes).
 * A job whose row differs from current_alloc[j] while current_alloc[j] holds
 * at least one GPU is multiplied by (T_j - R_j*delta)/(T_j + delta).  A job
 * with K = 0 or no feasible grid point has goodput and SPEEDUP 0.
 * fitness[c] = (sum_j w_j SPEEDUP_j^p / sum_j w_j)^(1/p)  (p = 0: weighted
 * geometric mean), with IEEE limits for SPEEDUP = 0 (p < 0 or p = 0 gives 0).
 * Constraint check ("Interference avoidance", Sec. 4.2, and node capacity):
 * V = sum_n max(0, d_n - 1) + sum_n max(0, sum_j A[c,j,n] - node_capacity[n]),
 * d_n = number of jobs with nodes >= 2 and A[c,j,n] > 0; when V > 0 the
 * fitness is replaced by -V unless PX_FLAG_NO_CONSTRAINT_CHECK is set.
 *
 * With PX_FLAG_SAMPLE_M the maximum of Eq. 13 is taken the way Sec. 4.3
 * describes instead: for each candidate total batch size M = m_grid[j,i] > 0,
 * s = ceil(M / (K * m_mem)) - 1 is the smallest accumulation count whose per-GPU
 * batch m = ceil(M / (K * (s+1))) does not exceed m_mem = trunc(PX_M_MEM); the
 * point is skipped when s > Gs-1 or when the batch actually run, K*m*(s+1)
 * (M rounded up to a multiple of K*(s+1)), falls outside [M0, M_max]; the best
 * of the remaining points is reported (best_m = m, best_s = s), ties to the
 * lowest i.  The fair-share goodput is found the same way.  Everything else is
 * unchanged.  Not available with precision 1 (PX_E_INVALID_ARG).
 *
 * fp64 (precision 0): best_goodput, speedup and fitness agree with a plain
 * fp64 evaluation of the formulas to a few units in the last place.
 * fp32 (precision 1): parameters are rounded to fp32 and all model arithmetic
 * is fp32; outputs are still stored as fp64.
 */
int pollux_fitness(const pollux_dims *dims,              /* host */
                   const int32_t *population,            /* [P,J,N] */
                   const double *job_params,             /* [PX_NPARAM,J] */
                   const int32_t *m_grid,                /* [J,Gm], values >= 1, duplicates allowed */
                   const int32_t *fair_share,            /* [J,2] = (GPUs, nodes) of the fair share */
                   const int32_t *current_alloc,         /* [J,N] */
                   const int32_t *node_capacity,         /* [N] */
                   double p, double delta,               /* fairness knob; re-allocation delay [s], >= 0 */
                   void *workspace, size_t workspace_bytes,
                   double *fitness,                      /* [P] out */
                   int32_t *best_m,                      /* [P,J] out: m* (the batch size, not its index), -1 if none;
                                                            may be NULL together with best_s (a search needs only fitness) */
                   int32_t *best_s,                      /* [P,J] out: s*, -1 if none; NULL exactly when best_m is */
                   double *best_goodput,                 /* [P,J] out, may be NULL */
                   double *speedup,                      /* [P,J] out, may be NULL: SPEEDUP_j (Eq. 15) after the penalty */
                   int32_t *violations,                  /* [P] out, may be NULL: V */
                   void *hip_stream);

/*
 * pollux_fitness with two HIP events (hipEvent_t cast to void*, created by the caller, both
 * required) recorded on the call's stream immediately before and immediately after the
 * grid-sweep kernel, the kernel that evaluates Eq. 4 over the (m, s) grid for every
 * (candidate, job) pair, so that a caller can time that kernel alone.  Everything else as
 * pollux_fitness.
 */
int pollux_fitness_timed(const pollux_dims *dims, const int32_t *population, const double *job_params,
                         const int32_t *m_grid, const int32_t *fair_share, const int32_t *current_alloc,
                         const int32_t *node_capacity, double p, double delta,
                         void *workspace, size_t workspace_bytes,
                         double *fitness, int32_t *best_m, int32_t *best_s, double *best_goodput, double *speedup,
                         int32_t *violations,
                         void *sweep_start_event, void *sweep_stop_event,   /* host handles */
                         void *hip_stream);

/*
 * pollux_fitness for callers that cannot allocate device memory or hand over a workspace: code
 * running under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The
 * same computation with the same kernels and the same results as pollux_fitness; the scratch
 * memory is an array of POLLUX_STATIC_SCRATCH_BYTES that is part of the library's code object
 * (every GPU the library runs on holds its own copy until the process ends).  The call
 * allocates and frees nothing.  Its first use on a device looks the array's address up (one
 * HIP runtime query, which may load the code object on that device); later calls only enqueue
 * kernels.
 *
 * Limit: pollux_workspace_size(dims) must not exceed POLLUX_STATIC_SCRATCH_BYTES, otherwise
 * PX_E_WORKSPACE is returned before anything is launched (64 MiB holds, for example, 1000
 * candidates x 200 jobs x 64 nodes with a 64 x 16 grid, which needs 46 MiB).
 *
 * Every call on a GPU uses that GPU's one array: two calls that overlap in time on one GPU
 * (different streams or threads) race and give undefined results; calls on one stream, or
 * otherwise ordered, are fine.  The array keeps what the last call left, so
 * PX_FLAG_KEEP_JOB_TABLES works as with a workspace of the caller's: the previous call through
 * this entry point on this GPU must then have had the same dims, job_params, m_grid, fair_share,
 * current_alloc, delta and other flags.  Without that flag the call itself clears what must
 * start at zero.
 *
 * status: device pointer to one int32, or NULL.  When given, the status word (PX_ST_* bits) of
 * this call is copied there on the stream after the last kernel; the host is not synchronised
 * (pollux_last_status does not apply: there is no workspace to name).
 * All other arguments, results and error codes as for pollux_fitness.
 */
#define POLLUX_STATIC_SCRATCH_BYTES (64u << 20)
int pollux_fitness_static(const pollux_dims *dims,       /* host */
                          const int32_t *population,     /* [P,J,N] */
                          const double *job_params,      /* [PX_NPARAM,J] */
                          const int32_t *m_grid,         /* [J,Gm] */
                          const int32_t *fair_share,     /* [J,2] */
                          const int32_t *current_alloc,  /* [J,N] */
                          const int32_t *node_capacity,  /* [N] */
                          double p, double delta,
                          double *fitness,               /* [P] out */
                          int32_t *best_m,               /* [P,J] out, may be NULL together with best_s */
                          int32_t *best_s,               /* [P,J] out, NULL exactly when best_m is */
                          double *best_goodput,          /* [P,J] out, may be NULL */
                          double *speedup,               /* [P,J] out, may be NULL */
                          int32_t *violations,           /* [P] out, may be NULL */
                          int32_t *status,               /* [1] out, may be NULL */
                          void *hip_stream);

typedef struct {
    uint64_t seed;           /* Philox key (low word, high word) */
    uint32_t generation;     /* counter word 0 */
    uint32_t elite_k;        /* survivors, 1..P: the best elite_k candidates are copied unchanged */
    uint32_t mut_threshold;  /* per-job mutation probability * 2^32, rounded down */
    uint32_t flags;          /* PX_GA_* */
    const int32_t *job_gpu_cap; /* device, [J], or NULL: the most GPUs job j may hold in a child (Sec. 4.1:
                                twice the most it has ever held); negative values count as 0 */
} pollux_ga_params;

enum {
    PX_GA_IN_PLACE = 1,  /* children == parents: child c (c >= elite_k) overwrites the candidate of rank c, which
                            did not survive, and the survivors stay where they are.  The new population holds the
                            same matrices as the out-of-place call, child c in slot order[c] instead of slot c,
                            and half of the traffic: survivors are neither read nor written. */
    PX_GA_INHERIT_ROWS = 2
                         /* pollux_generation only, with PX_GA_IN_PLACE: a row of a child that is a verbatim copy
                            of its parent's row (no move drawn for it, not touched by a repair) takes over the
                            parent's results for that row instead of being swept again: Eq. 13 sees a row only
                            through the job, its GPU count and whether it sits on one node, and the parent is a
                            survivor whose results the output arrays still hold.  Only the rows a move or a repair
                            has changed are read back and swept.  Results are what the call gives without the
                            flag; the work per generation drops from a sweep per (child, job) to a few per child. */
};

/*
 * One generation of the population search (Sec. 4.3: candidates are perturbed
 * and combined, then modified to satisfy node capacity and interference
 * avoidance).  The paper leaves the operators open; this library defines them
 * as follows, with every random draw taken from Philox4x32-10 (Salmon et al.,
 * SC'11), key = seed, counter = (generation, child, item, tag), word 0 unless
 * noted, and below(r, n) = (r * n) >> 32:
 *   rank     candidates ordered by (fitness descending, index ascending), NaN last;
 *   c < elite_k   child c = the candidate of rank c, verbatim;
 *   c >= elite_k  parents a, b = ranks below(word0, elite_k), below(word1, elite_k), and b = a when
 *                 bit 0 of word2 is set (a child of one parent)                       (item 0, tag 0);
 *                 row j comes from b if bit 0 is set, else from a                     (item j, tag 1);
 *                 if word0 < mut_threshold                                             (item j, tag 2)
 *                   then with move = word0 % 3 and x = word1                           (item j, tag 3),
 *                   occ = number of nodes on which the row is positive:
 *                   0 grow:   one more GPU on the below(x, occ)-th occupied node (ascending),
 *                             or on node below(x, N) if the job holds none;
 *                   1 shrink: one GPU less on the below(x, occ)-th occupied node (nothing if occ = 0);
 *                   2 pack:   row := 0 except row[below(x, N)] = min(sum of row, that node's capacity);
 *                 GPU limit (if job_gpu_cap is given, every row of a child, mutated or not): walking the
 *                   nodes in ascending order the job keeps its GPUs until job_gpu_cap[j] are kept; the
 *                   rest of the row is given back;
 *                 repair capacity: for each node over capacity, walking jobs cyclically
 *                   from below(word0, J) (item n, tag 4), remove GPUs until it fits;
 *                 repair interference: nodes in ascending order; of the multi-node jobs
 *                   present keep the one with most GPUs there (lowest j on ties), zero
 *                   the others there (their node counts drop, which later nodes see).
 * All arithmetic is integer; the result is a pure function of the arguments.
 *
 * dims: P, J, N and nothing else are read (Gm, Gs, precision and flags may hold anything, zero included);
 * the part of the workspace this call uses does not move with the grid, so it may share the workspace of
 * the pollux_fitness calls of a search, PX_FLAG_KEEP_JOB_TABLES included.  workspace_bytes must be at
 * least pollux_workspace_size of these dims with Gm and Gs taken as 1 when they are not positive.
 * Limit: the per-job and per-node bookkeeping of a child lives in the 160 KB of on-chip memory of a
 * compute unit: 16 N + 16 J + 12 E (+ 8 N if J < N, + 260 N if N <= 64) bytes, E = 1.5 J rounded up to a multiple of 256 and
 * kept within 512..3072, must not exceed 159 KB; beyond that PX_E_INVALID_ARG (e.g. J = 1000 jobs allow up to N = 5349 nodes).
 */
int pollux_ga_step(const pollux_dims *dims,              /* host; only P, J, N are read */
                   const int32_t *parents,               /* [P,J,N] */
                   const double *fitness,                /* [P] */
                   const int32_t *node_capacity,         /* [N] */
                   const pollux_ga_params *params,       /* host */
                   void *workspace, size_t workspace_bytes,
                   int32_t *children,                    /* [P,J,N] out, must not overlap parents; with
                                                            PX_GA_IN_PLACE it must equal parents */
                   void *hip_stream);

/*
 * One generation of the search in one call (Sec. 4.3): pollux_ga_step in place on `population`, ranking by
 * the values `fitness` holds, then pollux_fitness of the children the step has just formed, and of those
 * only.  A survivor's matrix is unchanged and FITNESS_p of a matrix depends on nothing else that changes
 * within a scheduling interval, so its entries of fitness, best_m, best_s, best_goodput, speedup and
 * violations are left as they are; the children's entries are overwritten.  After the call every output
 * array holds exactly what pollux_ga_step followed by a pollux_fitness call on the whole new population
 * would have left there, at the cost of sweeping P - elite_k candidates instead of P.
 *
 * Preconditions (as for PX_FLAG_KEEP_JOB_TABLES, which is implied): the previous call on this workspace was
 * pollux_fitness or pollux_generation with the same dims, job_params, m_grid, fair_share, current_alloc, p,
 * delta, flags and output arrays, and the output arrays and the population have not been written since.
 * params->flags must be PX_GA_IN_PLACE, optionally with PX_GA_INHERIT_ROWS (with PX_FLAG_MEMOISE in dims that
 * needs PX_FLAG_PAIR_RESULTS there too, in this call and in the calls before it).  The status word keeps
 * accumulating.
 * With PX_GA_INHERIT_ROWS a child whose matrix was formed the ordinary way (no negative entry met, every node
 * brought within its capacity, the per-node lists on chip large enough) satisfies both constraints by
 * construction and is given violations = 0 without its matrix being read again; any other child is evaluated in
 * full.
 * Errors as for pollux_fitness and pollux_ga_step.
 */
int pollux_generation(const pollux_dims *dims,           /* host */
                      int32_t *population,               /* [P,J,N] in/out */
                      const double *job_params,          /* [PX_NPARAM,J] */
                      const int32_t *m_grid,             /* [J,Gm] */
                      const int32_t *fair_share,         /* [J,2] */
                      const int32_t *current_alloc,      /* [J,N] */
                      const int32_t *node_capacity,      /* [N] */
                      double p, double delta,
                      const pollux_ga_params *params,    /* host */
                      void *workspace, size_t workspace_bytes,
                      double *fitness,                   /* [P] in/out */
                      int32_t *best_m,                   /* [P,J] in/out, may be NULL together with best_s */
                      int32_t *best_s,                   /* [P,J] in/out, NULL exactly when best_m is */
                      double *best_goodput,              /* [P,J] in/out, may be NULL */
                      double *speedup,                   /* [P,J] in/out, may be NULL */
                      int32_t *violations,               /* [P] in/out, may be NULL */
                      void *hip_stream);

/*
 * Online fitting of theta_sys (Sec. 4.1, "Online model fitting"): for each job the seven
 * throughput parameters (Eq. 12) that minimise the root mean squared logarithmic error
 * between Eq. 11 and the iteration times the job has recorded, subject to every alpha and
 * beta >= 0 and 1 <= gamma <= 10.  A record is (K, nodes, m, s, T_iter): GPUs and nodes of the
 * allocation it was measured on (what Eq. 9 sees of it), per-GPU batch size, accumulation
 * steps, seconds per iteration; record o of job j is element [j * max_obs + o] of each obs_*
 * array, o < obs_count[j] <= max_obs.  K >= 1, nodes >= 1, m >= 1, s >= 0, T_iter > 0 are the
 * caller's responsibility.
 * "Prior-driven exploration" (same section): the node pair alpha_sync^node, beta_sync^node is
 * held at 0 while the job has no record on more than one node, both beta_sync while it has
 * none with more than two GPUs, and all four sync parameters while it has none with more
 * than one GPU.
 * The minimiser is a box-constrained damped Gauss-Newton iteration, at most max_iter steps
 * (accepted or rejected) per starting point, one wavefront per job and starting point.  It starts from
 * theta_init[.,j] when theta_init is given, else from T_min = min_o T_o/(s_o+1) (first record on
 * ties): alpha_grad = T_min/2, beta_grad = T_min/(2 m at that record), alpha_sync = T_min/10,
 * beta_sync = T_min/100, gamma = 2.  The error has several local minima; with n_starts > 1 (at
 * most 5) further starts are tried and the best end point is kept (the earliest on ties): starts 2
 * and 3 first minimise with gamma held at 1 (where Eq. 11 is linear in the alphas and betas) and then
 * release gamma from 2 and from 5; starts 4 and 5 scale the four sync parameters by 3 and 0.3 and
 * begin at gamma = 1.2 and 5.  In every start, a sync pair (alpha, beta) that ends at zero, where the
 * error does not depend on it when gamma > 1, is put back to T_min/10 once and the iteration continued;
 * the better of the two end points is kept.
 * theta[i*J + j] is parameter i of job j in the order PX_ALPHA_G .. PX_GAMMA, i.e. the first
 * seven rows of job_params; rmsle[j] is the error reached; iterations[j] the steps taken over
 * all starting points.
 * A job without records gets theta = (0,0,0,0,0,0,1) and rmsle 0.
 * Returns PX_E_INVALID_ARG for null pointers (theta_init and iterations may be NULL), J < 1,
 * max_obs < 1, max_iter < 0 or n_starts outside 1..5.  No workspace; nothing is allocated.
 */
int pollux_fit_theta(int32_t J, int32_t max_obs,
                     const int32_t *obs_count,           /* [J] */
                     const int32_t *obs_K,               /* [J,max_obs] */
                     const int32_t *obs_nodes,           /* [J,max_obs] */
                     const int32_t *obs_m,               /* [J,max_obs] */
                     const int32_t *obs_s,               /* [J,max_obs] */
                     const double *obs_T,                /* [J,max_obs] seconds */
                     const double *theta_init,           /* [7,J] or NULL */
                     int32_t max_iter, int32_t n_starts,
                     double *theta,                      /* [7,J] out */
                     double *rmsle,                      /* [J] out */
                     int32_t *iterations,                /* [J] out, may be NULL */
                     void *hip_stream);

/*
 * Goodput-based auto-scaling (Sec. 5.3.3, "Cloud auto-scaling"), in two calls.
 *
 * pollux_goodput_per_gpu: per_gpu[j*(max_nodes+1) + 0] = max over (m, s) of GOODPUT of job j on one GPU, the
 * "predicted ideal goodput assuming perfect scalability" per GPU; per_gpu[j*(max_nodes+1) + n], n = 1..max_nodes,
 * = max over (m, s) of GOODPUT on n full nodes (K = n * gpus_per_node GPUs on n nodes) divided by K.  The
 * maximum is the one of Eq. 13 over the same grid as pollux_fitness (dims->Gm, dims->Gs, m_grid); dims->P and
 * dims->N only size the workspace (pollux_workspace_size(dims)) and may be 1; precision 0 and flags 0 only.
 *
 * pollux_autoscale: job j, now on nodes_now[j] nodes, scales up when per_gpu[j][nodes_now[j]] > U * per_gpu[j][0];
 * nodes are then added one at a time while the next count still has per_gpu >= L * per_gpu[j][0] and does not
 * exceed max_nodes.  Otherwise (or with nodes_now[j] outside 1..max_nodes) nodes_new[j] = nodes_now[j].  The
 * paper uses U = 2/3, L = 1/2.
 */
int pollux_goodput_per_gpu(const pollux_dims *dims,      /* host */
                           const double *job_params,     /* [PX_NPARAM,J] */
                           const int32_t *m_grid,        /* [J,Gm] */
                           int32_t gpus_per_node, int32_t max_nodes,
                           void *workspace, size_t workspace_bytes,
                           double *per_gpu,              /* [J,max_nodes+1] out */
                           void *hip_stream);
int pollux_autoscale(int32_t J, int32_t max_nodes,
                     const double *per_gpu,              /* [J,max_nodes+1] */
                     const int32_t *nodes_now,           /* [J] */
                     double U, double L,
                     int32_t *nodes_new,                 /* [J] out */
                     void *hip_stream);

/*
 * One interval of a discrete-time simulation of the jobs (Sec. 5.3, "Simulator construction", "Simulator
 * fidelity"; the paper replays measured profiles, this call replays the goodput model itself).  Job j holds
 * K[j] GPUs on nodes[j] nodes.  Its goodput[j] is the maximum of Eq. 13 there (the batch size and
 * accumulation steps its agent would choose), 0 if K[j] = 0 or the job has finished; its progress[j]
 * (in/out, examples at the efficiency of the initial batch size) advances by
 * goodput[j] * (dt - restart_delay if changed[j] != 0), never backwards; finished[j] = progress[j] >= target[j].
 * dims as for pollux_goodput_per_gpu.
 */
int pollux_sim_tick(const pollux_dims *dims,             /* host */
                    const double *job_params,            /* [PX_NPARAM,J] */
                    const int32_t *m_grid,               /* [J,Gm] */
                    const int32_t *K,                    /* [J] */
                    const int32_t *nodes,                /* [J] */
                    const int32_t *changed,              /* [J] allocation changed in this interval */
                    const double *target,                /* [J] */
                    double dt, double restart_delay,     /* seconds; the paper injects 30 s per re-allocation */
                    void *workspace, size_t workspace_bytes,
                    double *progress,                    /* [J] in/out */
                    double *goodput,                     /* [J] out */
                    int32_t *finished,                   /* [J] out */
                    void *hip_stream);

/*
 * The end of a scheduling interval (Sec. 4.3: the allocation matrix of highest fitness is applied): picks the
 * best candidate, the first in the order of pollux_ga_step's ranking (fitness descending, index ascending, NaN
 * last), writes its index to best[0] and its matrix over current_alloc, and reports per job what the jobs'
 * agents and pollux_sim_tick need: K[j] = GPUs, nodes[j] = nodes with at least one GPU, changed[j] = 1 when the
 * job's row differs from its previous row in current_alloc and that previous row held at least one GPU (the
 * jobs that pay the re-allocation delay, Sec. 4.2).  dims: P, J, N are read.  No workspace.
 */
int pollux_apply_best(const pollux_dims *dims,           /* host */
                      const int32_t *population,         /* [P,J,N] */
                      const double *fitness,             /* [P] */
                      int32_t *current_alloc,            /* [J,N] in/out */
                      int32_t *best,                     /* [1] out */
                      int32_t *K,                        /* [J] out */
                      int32_t *nodes,                    /* [J] out */
                      int32_t *changed,                  /* [J] out */
                      void *hip_stream);

/* Copies the status word of the last pollux_fitness (or pollux_fitness_timed) call that used `workspace`
 * to *host_out.  Synchronises `hip_stream`.  pollux_goodput_per_gpu and pollux_sim_tick neither clear nor
 * set the word; they do rewrite the job tables of the workspace, so a pollux_fitness call with
 * PX_FLAG_KEEP_JOB_TABLES may follow them only if they were given the same job_params, m_grid and grid. */
int pollux_last_status(const void *workspace, void *hip_stream, int32_t *host_out /* host */);

/* Text for a PX_* return code (static storage, never NULL). */
const char *pollux_strerror(int code);

/* POLLUX_VERSION of the built library. */
int pollux_version(void);

#ifdef __cplusplus
}
#endif
#endif /* POLLUX_H */
