// Fitness evaluation of a population of allocation matrices on gfx950.
//
// Pollux (arXiv 2008.12260): goodput model Sec. 3 (Eq. 4), statistical
// efficiency Sec. 3.1 (Eq. 6), throughput Sec. 3.2 (Eq. 7-11), per-job tuning
// Sec. 4.1 (Eq. 13), SPEEDUP / FITNESS_p, re-allocation penalty and
// interference avoidance Sec. 4.2 (Eq. 14-15).
//
// Kernels (one call = five launches on the caller's stream)
//   tables_kernel     per job and grid point: T_grad(m) (Eq. 8), 1/T_grad, ln T_grad, phi/m and
//                     the feasibility bounds; reciprocals; the largest node capacity; clears the status
//                     word and the per-node counters
//   last_kernel       per job, placement class and GPU count K <= 64 (one wavefront
//                     per eight rows; the "one node" class only up to the largest node capacity):
//                     T_sync (Eq. 9) and, for every batch size of the grid, the last pass of Eq. 10,
//                     (T_grad^g + T_sync^g)^(1/g), and the two terms C and A0 the sweep needs of it.
//                     They depend on the allocation only through K and on whether the job sits on
//                     one node, so they are shared by the population;
//                     also the feasible accumulation counts per (job, K, batch size)
//   jobs_kernel       per job (one wavefront): parameter checks, restart factor,
//                     fair-share goodput (denominator of Eq. 15)
//   pairs_kernel      per (candidate, job) (one wavefront): row reduce, sweep of the
//                     (m, s) grid, argmax; the row's non-zero entries are added to
//                     per-candidate, per-node counters with integer atomics
//   candidates_kernel per candidate (one workgroup): SPEEDUP, penalty, constraint
//                     check from those counters and the generalized mean
// With PX_FLAG_MEMOISE, memo_kernel sweeps once per (job, placement class, K <= 64) and the population pass looks
// the result up: pairs_kernel, or for rows of 65 to 256 nodes memo_candidates_kernel, which takes a whole candidate
// per workgroup and finishes its fitness as well (no per-pair scratch, no candidates_kernel).
// With PX_FLAG_SAMPLE_M the sweep is replaced by sweep_sampled (Sec. 4.3), the kernels
// instantiated with CH = 0, and last_kernel is not launched.
// For pollux_generation the population pass takes a list of candidates (the children of the search step), or,
// with PX_GA_INHERIT_ROWS, per job the list of rows the step has changed, after inherit_kernel has given every
// unchanged row the results of the row it was copied from.
//
// How one wavefront sweeps the grid of a (candidate, job) pair.  Lane l owns
// the batch sizes m_i, i = l, l+64, ...; it walks s = 0..Gs-1.  Dividing Eq. 4
// through by M gives
//     GOODPUT = (phi + M0) / h,   h(m, s) = T_iter(m, s) * (1 + phi / M),
// and with u = phi/(K m), last = (T_grad^g + T_sync^g)^(1/g):
//     h(m, s) = (last + u T_grad) + s T_grad + (last - T_grad) u / (s + 1)
//             = A0 + T_grad w(s),    w(s) = s + C / (s + 1),   C = (last - T_grad) u / T_grad,
// with every term non-negative.  The argmax of GOODPUT is the argmin of h over the
// feasible points.  For one batch size (one lane) that is the argmin of w over its
// feasible s, which form an interval s_lo..s_hi that depends on (job, K, m) only and is
// tabled.  The lane scans w over ALL s, one fused multiply-add per grid point; the four values
// of a group of four consecutive s are reduced with three v_min_f64, and the running minimum takes
// that result after its low five mantissa bits have been replaced by the first position of the group (so
// the minimum carries the group it came from and equal values resolve to the earlier group; the
// perturbation is 2^-47 relative).  The s inside the winning group is found once per lane
// afterwards by an exact comparison: w(s+1) < w(s) precisely when C > (s+1)(s+2), so the argmin is
// a count of thresholds below C (scan_argmin; equal values: the smaller s).  w is convex in s
// (C >= 0), so the feasible optimum sits at the scan's argmin clamped to s_lo..s_hi; h is
// formed there once per lane and group of 64 batch sizes.  The wave then takes the
// smallest h (equal values: lowest flat index), and the elected point is evaluated
// again with the formulas in the paper's own order (separate multiply and add, IEEE
// division), so the reported goodput does not depend on the fast form.
//
// The last pass of Eq. 10 is evaluated as
//     max(Tg, Ts) * exp( log1p( exp(-g |ln Tg - ln Ts|) ) / g ),
// which is the same quantity with the larger term factored out: every
// intermediate stays in [0, ln 2] or [1, 2], so plain fp64 log/exp give a result
// within a few ulp, where a direct pow(pow + pow, 1/g) would need an extended
// precision logarithm.  T_sync = 0 and g = 1 are taken exactly (T_grad and the
// plain sum).

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/pollux.h"
#include "pollux_device.h"
#include "pollux_host.h"
#include "pollux_math.h"

namespace px {

constexpr int kWavesPerBlock = 4;
constexpr int kMaxCandPerWave = 16;   // pairs kernel: candidates one wavefront walks at most (lane r keeps what candidate r needs)
constexpr int kRecipTable = 256;      // 1/K is tabled for K below this

// Result of the sweep for one (job, placement class, K); filled and used only in memoised mode.
struct __align__(16) MemoEntry {
    double goodput;
    int32_t m, s;
};

struct FitnessArgs {
    int P, J, N, Gm, Gs, flags;
    int cand_per_wave, cand_groups;   // pairs kernel: candidates each wavefront walks, groups of 4 * cand_per_wave
    const int32_t *population, *m_grid, *fair_share, *current_alloc, *node_capacity;
    const double *job_params;
    double p, delta;
    // workspace
    int32_t *status;
    double *rs, *rk, *lntg, *pu, *qh5, *ql5, *lt, *denom, *factor, *G;
    float *rsf;                   // 1/(s+1) in fp32, as long as rs
    double2 *tg;                  // [J,Gm] (T_grad, 1 / T_grad)
    double2 *ca;                  // [J,2,kTableK,Gm] (C, A0) of the sweep per (job, one node?, K, grid point) (see last_kernel)
    int32_t *srange;              // [J,kTableK,Gm] feasible accumulation counts per (job, K, grid point) (see last_kernel)
    int32_t *k1;                  // one word: the rows of the "one node" class are tabled for K <= *k1 only (tables_kernel)
    int gs_pad;                   // Gs rounded up to a multiple of 32: length of rs
    int32_t *running, *meta;
    MemoEntry *memo;              // [J,2,kTableK] best point per (job, one node?, K), memoised mode only
    int32_t *redo;                // [P] memoised mode: candidates left to the second instance of memo_candidates_kernel
    unsigned long long *curmask;  // [J] rows of at most 256 entries in 16-byte groups: bit g set when group g of the job's
                                  // current row holds a non-zero entry (jobs_kernel)
    int32_t *zeros;               // 64 zero bytes (jobs_kernel): what lanes read where the current row holds nothing
    unsigned long long *colpack;  // [P,N] per node: GPUs asked (low 40 bits, signed) + multi-node jobs present << 40
    int need_constraints;
    const int32_t *sel;           // candidates to evaluate (device list of n_sel indices into the population), or null: all P
    int n_sel;
    // row inheritance (pollux_generation with PX_GA_INHERIT_ROWS; written by the search step, see GaArgs)
    const int32_t *src_row;       // [n_sel, J] the candidate whose row j the listed child holds unchanged, or -1
    const int32_t *odd;           // [n_sel] the listed child is to be evaluated in full
    int32_t *dirty_count, *dirty; // rows to sweep, per job: their number [J] and the candidates they belong to [J, n_sel]
    int clear_status;             // tables_kernel starts a new status word (fitness calls; the query calls leave it alone)
    int clear_counters;           // tables_kernel clears colpack (fitness calls whose population pass keeps the counters in memory)
    // outputs
    double *fitness, *best_goodput, *speedup;
    int32_t *best_m, *best_s, *violations;
};

constexpr unsigned long long kPackJob = 1ull << 40;   // one multi-node job in a colpack word
constexpr int kNearRecips = 256;          // pairs kernel: reciprocals kept in LDS when Gs (rounded up to 32) is at most this
// The fp64 table in LDS (in doubles): per count s the pair (1 / (s + 1), s), so that one read brings both operands of
// w(s) = s + C / (s + 1) at the clamped count; behind the pairs the thresholds U[t] = t (t + 1).
constexpr int kNearU = 2 * kNearRecips;
// pairs kernel: the table rows (one per (placement class, K)) that most of a workgroup's pairs read are staged in LDS,
// behind the reciprocals and thresholds: (T_grad, 1 / T_grad) per batch size as in memory, then per row the (C, A0)
// pairs and the feasible ranges.  16-byte entries throughout, so that a lane's addresses are its number times 16
// (or times 4 for the ranges) plus a uniform offset, as they are for the tables in memory.
constexpr int kStageGm = 128;             // staged rows hold grids of at most this many batch sizes
constexpr int kStageRows = 4;             // rows staged at most (16.6 KB of LDS per workgroup with the rest: eight workgroups per CU)
constexpr int kStageRowDoubles = 2 * kStageGm + kStageGm / 2;
constexpr int kStageBase = kNearU + kNearRecips + 8;
constexpr int kStageDoubles = 2 * kStageGm + kStageRows * kStageRowDoubles;
constexpr int kPending = -2;             // pairs kernel: grid index of a row whose sweep is still to be done
constexpr int kMetaChanged = 1 << 30;   // meta[pair] = nodes | (row differs from current ? kMetaChanged : 0)

// Parameters of one job (uniform across the wavefront).  The sweep itself needs only
// phi and a = phi + M0; the synchronisation parameters are read where T_sync is formed.
struct Job {
    const double *__restrict__ jp;   // job_params
    int J, j;
    double phi, a;
};

struct SyncParams {
    double alpha_sl, beta_sl, alpha_sn, beta_sn, gamma, inv_gamma;
};

__device__ __forceinline__ Job load_job(const double *__restrict__ jp, int J, int j)
{
    Job q;
    q.jp = jp; q.J = J; q.j = j;
    q.phi = jp[(size_t)PX_PHI * J + j];
    q.a = q.phi + jp[(size_t)PX_M0 * J + j];
    return q;
}

__device__ __forceinline__ SyncParams load_sync(const Job &q)
{
    SyncParams y;
    y.alpha_sl = q.jp[(size_t)PX_ALPHA_SL * q.J + q.j];
    y.beta_sl = q.jp[(size_t)PX_BETA_SL * q.J + q.j];
    y.alpha_sn = q.jp[(size_t)PX_ALPHA_SN * q.J + q.j];
    y.beta_sn = q.jp[(size_t)PX_BETA_SN * q.J + q.j];
    y.gamma = q.jp[(size_t)PX_GAMMA * q.J + q.j];
    y.inv_gamma = 1.0 / y.gamma;
    return y;
}

// ---- tables ------------------------------------------------------------------
// Per job and grid point i (batch size m = m_grid[j,i]):
//   tg   = (T_grad(m), 1 / T_grad(m)) (Eq. 8)          lntg = ln T_grad(m)
//   pu   = phi / m                      (u = phi / (K m) = pu / K)
//   qh5  = floor(M_max / m) + 1/2       ql5  = ceil(M0 / m) - 1/2
// M0 <= K m (s+1) <= M_max holds exactly when ceil(M0/m) <= K (s+1) <= floor(M_max/m),
// i.e. for s between trunc(ql5 / K) and trunc(qh5 / K) - 1; the halves keep the
// quotients at least 1/(2K) away from an integer, so a rounded 1/K cannot move them
// across one.  Also rs[s] = 1/(s+1), rk[K] = 1/K, and a fitness call clears the status word here.
__global__ void __launch_bounds__(256) tables_kernel(FitnessArgs a)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t == 0 && a.clear_status) *a.status = 0;
    if (blockIdx.x == 0) {
        // A job that sits on one node holds at most that node's GPUs, so the tables of the "one node" class stop at
        // the largest capacity (all of kTableK when the call names no capacities); a row that claims more on one
        // node, which no valid allocation does, is swept in place like a row beyond the tables.
        __shared__ int cap_lds[256];
        int c = 0;
        if (a.node_capacity) {
            for (int n = threadIdx.x; n < a.N; n += 256) {
                const int v = a.node_capacity[n];
                c = v > c ? v : c;
            }
        }
        cap_lds[threadIdx.x] = c;
        __syncthreads();
        for (int half = 128; half > 0; half >>= 1) {
            if ((int)threadIdx.x < half) cap_lds[threadIdx.x] = cap_lds[threadIdx.x] > cap_lds[threadIdx.x + half] ? cap_lds[threadIdx.x] : cap_lds[threadIdx.x + half];
            __syncthreads();
        }
        if (threadIdx.x == 0) *a.k1 = (a.node_capacity && cap_lds[0] < kTableK) ? cap_lds[0] : kTableK;
    }
    const int rs_len = ((a.Gs + 31) / 32) * 32;
    if (t < rs_len) {
        a.rs[t] = 1.0 / (double)(t + 1);
        a.rsf[t] = 1.0f / (float)(t + 1);
    }
    if (t < kRecipTable) a.rk[t] = t > 0 ? 1.0 / (double)t : 0.0;
    if (a.clear_counters) {
        // the per-candidate, per-node counters of the constraint check start the call at zero
        const size_t n = (size_t)a.P * a.N;
        for (size_t i = (size_t)t; i < n; i += (size_t)gridDim.x * blockDim.x) a.colpack[i] = 0ull;
    }
    if (t < a.J * a.Gm) {
        const int j = t / a.Gm;
        const int mi = a.m_grid[t];
        const double m = (double)mi;
        const double tg = a.job_params[(size_t)PX_ALPHA_G * a.J + j] + a.job_params[(size_t)PX_BETA_G * a.J + j] * m;   // Eq. 8
        a.tg[t] = double2{tg, tg > 0.0 ? 1.0 / tg : 0.0};
        a.lntg[t] = px_log(tg);
        double qh = -1.5, ql = 1.0;
        if (mi > 0) {
            const double Mmax = a.job_params[(size_t)PX_MMAX * a.J + j], M0 = a.job_params[(size_t)PX_M0 * a.J + j];
            qh = floor(Mmax / m);
            if (m * (qh + 1.0) <= Mmax) qh += 1.0;
            if (m * qh > Mmax) qh -= 1.0;
            ql = ceil(M0 / m);
            if (m * (ql - 1.0) >= M0) ql -= 1.0;
            if (m * ql < M0) ql += 1.0;
            if (!(ql >= 1.0)) ql = 1.0;
            if (!(qh >= 0.0)) qh = -1.5;
        }
        a.pu[t] = mi > 0 ? a.job_params[(size_t)PX_PHI * a.J + j] / m : 0.0;
        a.qh5[t] = qh + 0.5;
        a.ql5[t] = ql - 0.5;
    }
}

// ---- T_sync and the last pass of Eq. 10 ------------------------------------------

// Eq. 9: no synchronisation for one GPU, the "local" pair on one node, the "node" pair otherwise.
__device__ __forceinline__ double t_sync(const SyncParams &y, int K, bool one_node)
{
    if (K <= 1) return 0.0;
    return one_node ? y.alpha_sl + y.beta_sl * (double)(K - 2) : y.alpha_sn + y.beta_sn * (double)(K - 2);
}

struct SyncTerm {
    double ts, lnts, gamma, inv_gamma;
    int mode;           // 0: T_sync = 0 (last pass = T_grad); 1: gamma = 1 (plain sum); 2: general
};

__device__ __forceinline__ SyncTerm sync_term(const Job &q, int K, bool one_node)
{
    const SyncParams y = load_sync(q);
    SyncTerm t;
    t.ts = t_sync(y, K, one_node);
    t.gamma = y.gamma;
    t.inv_gamma = y.inv_gamma;
    t.mode = (t.ts == 0.0) ? 0 : (y.gamma == 1.0 ? 1 : 2);
    t.lnts = (t.mode == 2) ? px_log(t.ts) : 0.0;
    return t;
}

__device__ __forceinline__ double last_pass(const SyncTerm &t, double tg, double lntg)
{
    if (t.mode == 0) return tg;
    if (t.mode == 1) return tg + t.ts;
    const double e = px_exp(-t.gamma * fabs(lntg - t.lnts));
    return fmax(tg, t.ts) * px_exp(px_log1p_unit(e) * t.inv_gamma);
}

// The feasible accumulation counts of grid point i with K GPUs: s_lo <= s <= s_hi
// (empty when s_lo > s_hi), from the half-offset quotients of tables_kernel.
__device__ __forceinline__ void feasible_range(double ql5, double qh5, double rK, int Gs, int &s_lo, int &s_hi)
{
    s_lo = (int)(ql5 * rK);
    s_hi = (int)(qh5 * rK) - 1;
    s_hi = s_hi < Gs - 1 ? s_hi : Gs - 1;
}

// Whether the tables hold the row of (K, class): K = 1 .. kTableK for several nodes, 1 .. k1 for one node.
__device__ __forceinline__ bool tabled_row(int K, bool one_node, int k1)
{
    return K <= (one_node ? k1 : kTableK);
}

// lt[row][i] for every grid point i, row index ((j * 2 + one_node) * kTableK + (K - 1)).
// One wavefront fills kLastRows rows of one (job, placement class): their inputs are read once and lane r
// prepares T_sync and its logarithm for the r-th of them.  The rows of the "several nodes"
// class also write the feasible accumulation counts of (job, K, i), which do not depend on
// the class: srange[j][K-1][i] = first | last << 16, first > last when there is none.
// Beside lt[row][i] the wavefront writes ca[row][i] = (C, A0), the two terms the sweep needs of (job, class, K, i):
//     h(m_i, s) = A0 + T_grad (s + C / (s + 1)),   u = phi / (K m_i),   A0 = last + u T_grad,   C = (last - T_grad) u / T_grad,
// formed here once instead of by every (candidate, job) pair; A0 = +inf where no accumulation count is feasible, so
// such a batch size never wins an election.
constexpr int kLastRows = 8;
static_assert(kTableK % kLastRows == 0, "the rows of a wavefront belong to one job and class");

__device__ __forceinline__ double wave_read(double v, int src)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), src), __builtin_amdgcn_readlane(__double2loint(v), src));
}

__global__ void __launch_bounds__(256) last_kernel(FitnessArgs a)
{
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long row0 = ((long long)blockIdx.x * kWavesPerBlock + wave) * kLastRows;
    if (row0 >= (long long)a.J * 2 * kTableK) return;
    const int K0 = (int)(row0 % kTableK) + 1;
    const bool one_node = ((row0 / kTableK) & 1) != 0;
    const int j = (int)(row0 / (2 * kTableK));
    if (one_node && K0 > *a.k1) return;             // no row of this wavefront is ever looked up
    const Job q = load_job(a.job_params, a.J, j);
    const int lane = lane_id();
    const SyncTerm mine = sync_term(q, K0 + (lane < kLastRows ? lane : 0), one_node);
    SyncTerm t[kLastRows];
#pragma unroll
    for (int r = 0; r < kLastRows; ++r) {
        t[r].ts = wave_read(mine.ts, r);
        t[r].lnts = wave_read(mine.lnts, r);
        t[r].gamma = mine.gamma;
        t[r].inv_gamma = mine.inv_gamma;
        t[r].mode = __builtin_amdgcn_readlane(mine.mode, r);
    }
    double rK[kLastRows];
#pragma unroll
    for (int r = 0; r < kLastRows; ++r) rK[r] = a.rk[K0 + r];
    const size_t o = (size_t)j * a.Gm;
    int32_t *__restrict__ out = a.srange + ((size_t)j * kTableK + (size_t)(K0 - 1)) * a.Gm;
    for (int i = lane; i < a.Gm; i += kWave) {
        const double2 tgr = a.tg[o + i];
        const double tg = tgr.x, lntg = a.lntg[o + i], pu = a.pu[o + i];
        const double ql5 = a.ql5[o + i], qh5 = a.qh5[o + i];
#pragma unroll
        for (int r = 0; r < kLastRows; ++r) {
            const double last = last_pass(t[r], tg, lntg);
            a.lt[(size_t)(row0 + r) * a.Gm + i] = last;
            int s_lo, s_hi;
            feasible_range(ql5, qh5, rK[r], a.Gs, s_lo, s_hi);
            const bool none = s_lo > s_hi || s_hi < 0;
            if (none) { s_lo = 1; s_hi = 0; }
            if (!one_node) out[(size_t)r * a.Gm + i] = s_lo | (s_hi << 16);
            // what the sweep needs of (job, class, K, i): h(m_i, s) = A0 + T_grad (s + C / (s+1))
            const double u = pu * rK[r];
            const double A0 = px_fma(u, tg, last);
            const double B0 = (last - tg) * u;
            a.ca[(size_t)(row0 + r) * a.Gm + i] = double2{B0 * tgr.y, none ? __builtin_inf() : A0};
        }
    }
}

// ---- the sweep of one (job, K, nodes) ----------------------------------------

struct Best {
    double goodput;   // maximum of Eq. 4 over the grid, 0 if nothing is feasible
    int m, s;         // batch size and accumulation steps attaining it, -1/-1 if none
};

struct JobTables {
    const int32_t *__restrict__ m;
    const double2 *__restrict__ tg;   // (T_grad, 1 / T_grad)
    const double *__restrict__ lntg, *__restrict__ pu, *__restrict__ qh5, *__restrict__ ql5;
    const double *__restrict__ lt;    // rows of this job in the last-pass table
    const double2 *__restrict__ ca;   // rows of this job in the table of (C, A0)
    const int32_t *__restrict__ srange;   // feasible accumulation counts of this job, [kTableK, Gm]
    int k1;                               // rows of the "one node" class are tabled for K <= k1
};

// Wave-wide argmax of non-negative goodput values g (0 = the lane has no point): positive
// doubles order like their bit patterns, so the maximum is found as two unsigned 32-bit
// reductions (high words, then low words among the lanes that hold the highest high word),
// and ties go to the lowest flat index.  Every lane returns the same result.
__device__ __forceinline__ Best wave_argmax(double g, int flat, int m, int s)
{
    g = g > 0.0 ? g : 0.0;                                        // also drops a NaN
    const unsigned hi = (unsigned)__double2hiint(g), lo = (unsigned)__double2loint(g);
    const unsigned hmax = wave_max(hi);
    const unsigned lmax = wave_max(hi == hmax ? lo : 0u);
    if ((hmax | lmax) == 0u) return Best{0.0, -1, -1};
    const bool top = hi == hmax && lo == lmax;
    const int fmin_ = wave_min(top ? flat : 0x7FFFFFFF);
    const uint64_t wmask = __ballot(top && flat == fmin_);
    const int wl = __builtin_amdgcn_readfirstlane(__ffsll((unsigned long long)wmask) - 1);
    Best out;
    out.goodput = __hiloint2double((int)__builtin_amdgcn_readfirstlane((int)hmax), (int)__builtin_amdgcn_readfirstlane((int)lmax));
    out.m = __builtin_amdgcn_readlane(m, wl);
    out.s = __builtin_amdgcn_readlane(s, wl);
    return out;
}

// Eq. 4 at one grid point, in the paper's order of operations (no contraction).
__device__ __forceinline__ double goodput_point(const Job &q, double Km, double tg, double last, int s)
{
    const double M = Km * (double)(s + 1);
    const double t_iter = (double)s * tg + last;                 // Eq. 11
    const double throughput = M / t_iter;                        // Eq. 7
    const double efficiency = q.a / (q.phi + M);                 // Eq. 6
    return throughput * efficiency;                              // Eq. 4
}

// ---- the sweep of one batch size per lane over CH accumulation counts ---------------
// With C = B0 / T_grad the quantity to minimise is  h = A0 + T_grad w(s),  w(s) = s + C / (s+1),
// for the lane's batch size.  The lane scans w over all accumulation counts, feasible or not;
// C >= 0 makes w convex in s, and the feasible counts of a batch size form an interval (tabled
// per (job, K, i) by last_kernel), so the smallest feasible w sits at the scan's argmin clamped
// to that interval (sweep_pick).  Inside a chunk of CH counts starting at s0, per group of four
// positions b = 4 G .. 4 G + 3 and lane:
//   w_b  = C * r + (b mod 16)  one v_fma_f64 each (v_mul_f64 for 0): r = 1/(s0 + b + 1) from scalar
//                              registers, the addend an inline constant (1, 2, 4) or one of
//                              twelve register pairs that hold 3, 5, 6, .. 15 for the whole kernel
//   g    = min of the four                                three v_min_f64
//   lo   = (31 & 4 G) | (~31 & lo(g))                     v_bfi_b32
//   kmin = min(kmin, key)                                 v_min_f64
// so the key carries its group's first position 4 G in the low five mantissa bits (equal values resolve to
// the earlier group): nine VALU instructions per four points; the reciprocals arrive through the
// scalar cache.  Each run of sixteen positions has a minimum of its own (values relative to
// the run's first position); the runs are merged after the chunk (merge_runs).  The position
// inside the winning group is found afterwards, once per lane (sweep_pick).
typedef const double __attribute__((address_space(4))) *ScalarDoubles;
typedef const double __attribute__((address_space(3))) *LdsDoubles;
typedef double Double2 __attribute__((ext_vector_type(2)));

constexpr int kRun = 16;
constexpr int runs_of(int CH) { return CH > kRun ? CH / kRun : 1; }
// Chunks of 16 and 32 tag per group of four positions; chunks of 8 tag every position (twelve instructions per
// four points, and less to find afterwards: quicker for very few counts per batch size).
constexpr bool grouped_tags(int CH) { return CH >= 16; }

// The addends that are not inline constants (3, 5 .. 15) in vector registers.  Made once
// per kernel through an opaque statement, so that they stay in registers instead of being formed
// again at every use.
struct RunSteps {
    double x[kRun];
};

__device__ __forceinline__ RunSteps make_run_steps()
{
    RunSteps X;
#pragma unroll
    for (int t = 0; t < kRun; ++t) X.x[t] = (double)t;
    asm volatile("" : "+v"(X.x[3]), "+v"(X.x[5]), "+v"(X.x[6]), "+v"(X.x[7]), "+v"(X.x[8]), "+v"(X.x[9]), "+v"(X.x[10]),
                      "+v"(X.x[11]), "+v"(X.x[12]), "+v"(X.x[13]), "+v"(X.x[14]), "+v"(X.x[15]));
    return X;
}

// w at position B of a chunk, relative to the first position of its run.
template <int B>
__device__ __forceinline__ double point_w(double C, double r, const RunSteps &X)
{
    constexpr int t = B % kRun;
    double g;
    if constexpr (t == 0) asm("v_mul_f64 %0, %1, %2" : "=v"(g) : "v"(C), "s"(r));
    else if constexpr (t == 1) asm("v_fma_f64 %0, %1, %2, 1.0" : "=v"(g) : "v"(C), "s"(r));
    else if constexpr (t == 2) asm("v_fma_f64 %0, %1, %2, 2.0" : "=v"(g) : "v"(C), "s"(r));
    else if constexpr (t == 4) asm("v_fma_f64 %0, %1, %2, 4.0" : "=v"(g) : "v"(C), "s"(r));
    else asm("v_fma_f64 %0, %1, %2, %3" : "=v"(g) : "v"(C), "s"(r), "v"(X.x[t]));
    return g;
}

// v with TAG in its low five mantissa bits.
template <int TAG>
__device__ __forceinline__ double tagged(double v)
{
    int lo;
    asm("v_bfi_b32 %0, 31, %1, %2" : "=v"(lo) : "n"(TAG), "v"(__double2loint(v)));
    return __hiloint2double(__double2hiint(v), lo);
}

// Four points at positions 4 G .. 4 G + 3 of the chunk (G a compile-time group index): the
// four values, their minimum, its key.  The volatile statements keep their order, so the
// reciprocals of a group are requested after the previous group's work and only one group's
// operands occupy scalar registers.
struct GroupRecips {
    double r0, r1, r2, r3;
};

template <int G>
__device__ __forceinline__ GroupRecips load_group(ScalarDoubles &rs)
{
    asm volatile("" : "+s"(rs));
    return GroupRecips{rs[4 * G + 0], rs[4 * G + 1], rs[4 * G + 2], rs[4 * G + 3]};
}

template <int CH, int G>
__device__ __forceinline__ void scan_group(double (&kmin)[runs_of(CH)], double C, const RunSteps &X, const GroupRecips &o)
{
    const double w0 = point_w<4 * G + 0>(C, o.r0, X);
    const double w1 = point_w<4 * G + 1>(C, o.r1, X);
    const double w2 = point_w<4 * G + 2>(C, o.r2, X);
    const double w3 = point_w<4 * G + 3>(C, o.r3, X);
    if constexpr (grouped_tags(CH)) {
        double g, g2;
        asm volatile("v_min_f64 %0, %2, %3\n\t"
                     "v_min_f64 %1, %4, %5\n\t"
                     "v_min_f64 %0, %0, %1"
                     : "=&v"(g), "=&v"(g2)
                     : "v"(w0), "v"(w1), "v"(w2), "v"(w3));
        const double key = tagged<4 * G>(g);         // the first position of the group: what scan_argmin wants of it
        if constexpr ((4 * G) % kRun == 0) kmin[4 * G / kRun] = key;      // the first group of a run starts its minimum
        else asm volatile("v_min_f64 %0, %0, %1" : "+v"(kmin[4 * G / kRun]) : "v"(key));
    } else {
        const double k0 = tagged<4 * G + 0>(w0), k1 = tagged<4 * G + 1>(w1), k2 = tagged<4 * G + 2>(w2), k3 = tagged<4 * G + 3>(w3);
        if constexpr ((4 * G) % kRun == 0) {
            asm volatile("v_min_f64 %0, %1, %2\n\t"
                         "v_min_f64 %0, %0, %3\n\t"
                         "v_min_f64 %0, %0, %4"
                         : "=&v"(kmin[4 * G / kRun])
                         : "v"(k0), "v"(k1), "v"(k2), "v"(k3));
        } else {
            asm volatile("v_min_f64 %0, %0, %1\n\t"
                         "v_min_f64 %0, %0, %2\n\t"
                         "v_min_f64 %0, %0, %3\n\t"
                         "v_min_f64 %0, %0, %4"
                         : "+v"(kmin[4 * G / kRun])
                         : "v"(k0), "v"(k1), "v"(k2), "v"(k3));
        }
    }
}

// The reciprocals of a group are requested one group ahead of their use.
template <int CH, int G = 0>
__device__ __forceinline__ void scan_groups(double (&kmin)[runs_of(CH)], double C, const RunSteps &X, ScalarDoubles &rs,
                                            GroupRecips cur)
{
    if constexpr (4 * G < CH) {
        asm volatile("" : "+s"(cur.r0), "+s"(cur.r1), "+s"(cur.r2), "+s"(cur.r3));
        GroupRecips next = cur;
        if constexpr (4 * (G + 1) < CH) next = load_group<G + 1>(rs);
        scan_group<CH, G>(kmin, C, X, cur);
        scan_groups<CH, G + 1>(kmin, C, X, rs, next);
    }
}

// min(lower, upper + D) for the minima of two neighbouring stretches of positions, the upper
// one starting D positions later; D is formed from inline constants.  The sum gets
// the group bits of `upper` back.
template <int D>
__device__ __forceinline__ double merge_runs(double lower, double upper)
{
    static_assert(D == 16, "an offset that is a product of inline constants");
    double moved;
    asm("v_fma_f64 %0, 4.0, 4.0, %1" : "=v"(moved) : "v"(upper));
    int lo;
    asm("v_bfi_b32 %0, 31, %1, %2" : "=v"(lo) : "v"(__double2loint(upper)), "v"(__double2loint(moved)));
    const double key = __hiloint2double(__double2hiint(moved), lo);
    double out;
    asm("v_min_f64 %0, %1, %2" : "=v"(out) : "v"(lower), "v"(key));
    return out;
}

// CH points starting at accumulation count s0; rs points at s0.  Returns the smallest key of
// w over the chunk (values relative to s0; in the low five bits the first position of the group of four, or the position).
template <int CH>
__device__ __forceinline__ double scan_chunk(double C, const RunSteps &X, ScalarDoubles rs)
{
    static_assert(CH == 8 || CH == 16 || CH == 32, "one or two runs");
    double kmin[runs_of(CH)];
    scan_groups<CH>(kmin, C, X, rs, load_group<0>(rs));
    if constexpr (runs_of(CH) == 1) return kmin[0];
    else return merge_runs<kRun>(kmin[0], kmin[1]);
}

// The same chunk for a GPU count beyond the tables, written as a plain loop (rare, so
// compactness counts more than speed): the lane's feasible positions are first..last.
template <int CH>
__device__ __forceinline__ double sweep_chunk_plain(double tg, double A0s, double B0, const double *__restrict__ rs,
                                                    int first, int last)
{
    double kmin = __builtin_inf();
#pragma unroll 1
    for (int b = 0; b < CH; ++b) {
        const double h = px_fma(B0, rs[b], px_fma((double)b, tg, A0s));
        const double key = __hiloint2double(__double2hiint(h), (__double2loint(h) & ~31) | b);
        if (first <= b && b <= last && key < kmin) kmin = key;
    }
    return kmin;
}

// The accumulation count with the smallest w(s) = s + C / (s + 1) among s = 0, 1, ... (all counts of the grid,
// rounded up to whole chunks: the reciprocals are padded), equal values to the lower count, for the lane's own C >= 0.
// near: a copy of the reciprocals in LDS with the thresholds U[t] = t (t+1) behind them, when has_near.
template <int CH>
__device__ __forceinline__ int scan_argmin(double C, const RunSteps &X, ScalarDoubles rsc, int Gs, LdsDoubles near, bool has_near)
{
    // the argmin of w over all counts (the first count of its group of four, where keys carry groups): low bits of the
    // smallest key, chunk by chunk
    double wmin = scan_chunk<CH>(C, X, rsc);
    int g_star = __double2loint(wmin) & 31;
    // (the bound goes through an opaque statement: every inlined copy of this loop then tests it with a scalar
    // comparison of its own, instead of sharing one truth value that the compiler carries around as a lane mask and
    // negates with two vector instructions)
    asm volatile("" : "+s"(Gs));
    for (int s0 = CH; s0 < Gs; s0 += CH) {
        const double w = scan_chunk<CH>(C, X, rsc + s0);
        const double moved = w + (double)s0;            // strictly smaller only: ties keep the smaller s
        if (moved < wmin) {
            wmin = moved;
            g_star = s0 + (__double2loint(w) & 31);
        }
    }
    // The keys of the scan carry index bits in their low mantissa bits, so what the scan has found is the
    // argmin up to values that agree to 2^-47; w is convex, so only neighbouring counts can agree that
    // closely, and the true argmin lies next to what the scan found.  The order of neighbours is known
    // exactly: w(s+1) < w(s) precisely when C > (s+1)(s+2), both sides exact in fp64.  With
    // U[t] = t (t+1) (U[0] = -1, so that the result never falls below 0) the argmin over all counts is the
    // number of t >= 0 with C > U[t], less one; only the t around the scan's result need to be looked at.
    int s_star;
    if constexpr (grouped_tags(CH)) {
        // the scan names a group of four counts 4 g .. 4 g + 3: the argmin is 4 g - 1 plus the number of
        // t = 4 g .. 4 g + 4 with C > U[t]
        const int t0 = g_star;
        s_star = t0 - 1;
        if (has_near) {
            // all five requested together: three reads in a row cost three LDS round trips per batch size, and after
            // the scan the registers its values occupied are free
            LdsDoubles u = near + kNearU + t0;
            const Double2 a01 = *(const Double2 __attribute__((address_space(3))) *)u;
            const Double2 a23 = *(const Double2 __attribute__((address_space(3))) *)(u + 2);
            const double a4 = u[4];
            s_star += (C > a01.x ? 1 : 0) + (C > a01.y ? 1 : 0);
            s_star += (C > a23.x ? 1 : 0) + (C > a23.y ? 1 : 0);
            s_star += C > a4 ? 1 : 0;
        } else {
            const double td = (double)t0;
            s_star += (C > (t0 > 0 ? px_fma(td, td, td) : -1.0) ? 1 : 0);
            s_star += (C > px_fma(td, td, px_fma(3.0, td, 2.0)) ? 1 : 0);
            s_star += (C > px_fma(td, td, px_fma(5.0, td, 6.0)) ? 1 : 0);
            s_star += (C > px_fma(td, td, px_fma(7.0, td, 12.0)) ? 1 : 0);
            s_star += (C > px_fma(td, td, px_fma(9.0, td, 20.0)) ? 1 : 0);
        }
    } else {
        // the scan names a count: one step down or up if its neighbour is better
        s_star = g_star;
        double t_lo, t_hi;
        if (has_near) {
            t_lo = near[kNearU + s_star];
            t_hi = near[kNearU + s_star + 1];
        } else {
            const double sd = (double)s_star;
            t_lo = s_star > 0 ? px_fma(sd, sd, sd) : -1.0;
            t_hi = px_fma(sd, sd, px_fma(3.0, sd, 2.0));
        }
        s_star = C <= t_lo ? s_star - 1 : (C > t_hi ? s_star + 1 : s_star);
    }
    return s_star;
}

// The grid point a sweep elects: index into the job's batch-size grid and accumulation
// count; i = -1 when no point is feasible.
struct Pick {
    int i, s;
};

// All 64 lanes call this with the same (job, K >= 1, nodes).  Every lane returns the same result:
// the feasible point with the smallest h over the whole grid (equal values resolve to the
// lowest flat index i * Gs + s).
// TABLED: last pass and feasible ranges come from the job's tables (K <= kTableK), else they are formed here.
// WHOLE: the caller has checked that Gm is a multiple of 64, so no lane runs past the grid of batch sizes.
template <int CH, bool TABLED, bool WHOLE = false>
__device__ __forceinline__ Pick sweep_pick(const Job &q, const JobTables &tb, const RunSteps &X, const double *__restrict__ rs,
                                           const double *__restrict__ rk, int Gm, int Gs, int K, int nodes,
                                           LdsDoubles near = nullptr, bool has_near = false, int staged_row = -1)
{
    // near: a copy of rs in LDS (quicker to read per lane) when has_near
    // staged_row: where in `near` the terms of this (class, K) are staged (TABLED and WHOLE; see kStageBase), or -1;
    // rows are staged only together with has_near
    const int lane = lane_id();
    K = __builtin_amdgcn_readfirstlane(K);        // the same in every lane (see above): kept in scalar registers
    nodes = __builtin_amdgcn_readfirstlane(nodes);
    // 1/K arrives through the scalar cache
    const double rK = K < kRecipTable ? ((ScalarDoubles)rk)[K] : 1.0 / (double)K;
    const bool one_node = nodes == 1;
    // offsets inside one job's tables fit 32 bits (Gm <= 2^20)
    const double2 *__restrict__ carow = tb.ca + (unsigned)((one_node ? kTableK : 0) + (TABLED ? K - 1 : 0)) * (unsigned)Gm;
    const int32_t *__restrict__ srow = tb.srange + (unsigned)(TABLED ? K - 1 : 0) * (unsigned)Gm;
    SyncTerm st = {0.0, 0.0, 1.0, 1.0, 0};
    if constexpr (!TABLED) st = sync_term(q, K, one_node);

    // where this lane's terms of a staged row start in LDS (bytes from `near`): the (C, A0) pairs, the feasible ranges
    const unsigned at_ca = ((unsigned)lane << 4) + 8u * (unsigned)staged_row;
    const unsigned at_range = ((unsigned)lane << 2) + 8u * (unsigned)(staged_row + 2 * kStageGm);

    double kbest = __builtin_inf();   // smallest h seen by this lane
    int where = 0;                    // its accumulation count | (index of its group of 64 batch sizes) << 16
    unsigned long long second = 0;    // staged terms: the lanes whose `where` belongs to the second group (no index in `where`)
    const ScalarDoubles rsc = (ScalarDoubles)rs;

    // One group of 64 batch sizes starting at i0.  G: the group's index when the terms are staged in LDS (the caller
    // stages only grids of one or two groups, so the index is a compile-time constant and the group's offset goes
    // into the LDS instructions' immediate fields), else -1.
    auto group = [&](const int i0, auto G) __attribute__((always_inline)) {
        constexpr int g = decltype(G)::value;
        const int i = i0 + lane;
        const bool active = WHOLE || i < Gm;
        const int il = active ? i : Gm - 1;
        // a uniform base plus a 32-bit byte offset per lane: the address needs no 64-bit vector arithmetic;
        // the offsets of the 16-byte and the 4-byte entries are one shift-and-add each on the lane number
        const unsigned at = (unsigned)il * 8u;
        // (the opaque statement keeps the two shifted counters on the scalar unit)
        unsigned i16 = (unsigned)i0 << 4, i4 = (unsigned)i0 << 2;
        asm("" : "+s"(i16), "+s"(i4));
        const unsigned at16 = WHOLE ? ((unsigned)lane << 4) + i16 : (unsigned)il * 16u;
        const unsigned at4 = WHOLE ? ((unsigned)lane << 2) + i4 : (unsigned)il * 4u;
        double key = __builtin_inf();    // h of this batch size at its best feasible count s_c
        int s_c = 0;
        bool feasible;
        if constexpr (TABLED) {
            double tg, C, A0;                        // A0 = +inf when the batch size has no feasible count
            int bounds;
            if constexpr (g >= 0) {
                // the row's offset is added to the lane's once per call; the group's is a constant
                typedef const char __attribute__((address_space(3))) *LdsBytes;
                const Double2 car = *(const Double2 __attribute__((address_space(3))) *)((LdsBytes)near + at_ca + 16 * kWave * g);
                C = car.x;
                A0 = car.y;
                tg = *(LdsDoubles)((LdsBytes)near + ((unsigned)lane << 4) + (8 * kStageBase + 16 * kWave * g));
                bounds = *(const int __attribute__((address_space(3))) *)((LdsBytes)near + at_range + 4 * kWave * g);
            } else {
                tg = *(const double *)((const char *)tb.tg + at16);
                const double2 car = *(const double2 *)((const char *)carow + at16);
                C = car.x;
                A0 = car.y;
                bounds = *(const int32_t *)((const char *)srow + at4);
            }
            const int s_lo = bounds & 0xFFFF, s_hi = bounds >> 16;
            feasible = active;
            // (rows are staged only in a workgroup that also keeps the table of reciprocals and thresholds in LDS)
            const bool tables_near = g >= 0 ? true : has_near;
            const int s_star = scan_argmin<CH>(C, X, rsc, Gs, near, tables_near);
            // convex w, feasible counts s_lo .. s_hi: the constrained argmin is the clamped one
            s_c = s_star < s_hi ? s_star : s_hi;
            s_c = s_c > s_lo ? s_c : s_lo;
            double r_c, sd_c;
            if (tables_near) {
                const Double2 rc = *(const Double2 __attribute__((address_space(3))) *)(near + 2 * s_c);
                r_c = rc.x;
                sd_c = rc.y;
            } else {
                r_c = *(const double *)((const char *)rs + 8u * (unsigned)s_c);
                sd_c = (double)s_c;
            }
            const double w_c = px_fma(C, r_c, sd_c);
            key = px_fma(tg, w_c, A0);
        } else {
            const double2 tgr = *(const double2 *)((const char *)tb.tg + 2u * at);
            const double tg = tgr.x;
            const double last = last_pass(st, tg, tb.lntg[il]);
            const double u = *(const double *)((const char *)tb.pu + at) * rK;
            const double A0 = px_fma(u, tg, last);
            const double B0 = (last - tg) * u;
            int s_lo = 1, s_hi = 0;
            feasible_range(tb.ql5[il], tb.qh5[il], rK, Gs, s_lo, s_hi);
            if (!active) s_hi = -1;
            for (int s0 = 0; s0 < Gs; s0 += CH) {
                const double A0s = s0 == 0 ? A0 : px_fma((double)s0, tg, A0);
                const double kmin = sweep_chunk_plain<CH>(tg, A0s, B0, rs + s0, s_lo - s0, s_hi - s0);
                if (kmin < key) {
                    key = kmin;
                    s_c = s0 + (__double2loint(kmin) & 31);
                }
            }
            feasible = key < __builtin_inf();
            if (feasible) {
                // the same exact order of neighbours as in the tabled path, inside the feasible counts; the key
                // is then formed again without index bits
                const double C = B0 * tgr.y, sd = (double)s_c;
                const double t_lo = px_fma(sd, sd, sd), t_hi = px_fma(sd, sd, px_fma(3.0, sd, 2.0));
                if (s_c > s_lo && C <= t_lo) s_c -= 1;
                else if (s_c < s_hi && C > t_hi) s_c += 1;
                key = px_fma(B0, rs[s_c], px_fma((double)s_c, tg, A0));
            }
        }
        if constexpr (g == 0) {
            // the first group starts the lane's minimum (a batch size without a feasible count has h = +inf)
            kbest = key;
            where = s_c;
        } else if constexpr (g == 1) {
            // which lanes hold a batch size of the second group stays a lane mask in scalar registers
            const bool better = key < kbest;
            second = __builtin_amdgcn_ballot_w64(better);
            kbest = better ? key : kbest;
            where = better ? s_c : where;
        } else if (feasible && key < kbest) {
            kbest = key;
            where = s_c | ((i0 / kWave) << 16);
        }
    };
    if (TABLED && WHOLE && staged_row >= 0) {
        group(0, std::integral_constant<int, 0>());
        if (Gm > kWave) group(kWave, std::integral_constant<int, 1>());
    } else {
        // the counter of this loop is advanced on the scalar unit (it would otherwise be copied to a vector register)
        for (int i0 = 0; i0 < Gm;) {
            group(i0, std::integral_constant<int, -1>());
            asm volatile("s_add_i32 %0, %0, 64" : "+s"(i0) : : "scc");
        }
    }

    // positive doubles order like their bit patterns: unsigned 32-bit wave minima, high words first;
    // the low words only among several lanes that share the smallest high word
    const unsigned hi = (unsigned)__double2hiint(kbest), lo = (unsigned)__double2loint(kbest);
    const unsigned hmin = wave_min(hi);
    if (hmin >= 0x7FF00000u) return Pick{-1, -1};              // every lane still holds +inf
    unsigned long long winners = __builtin_amdgcn_ballot_w64(hi == hmin);
    if (winners & (winners - 1)) {
        const unsigned lmin = wave_min(hi == hmin ? lo : 0xFFFFFFFFu);
        winners &= __builtin_amdgcn_ballot_w64(lo == lmin);
        if (winners & (winners - 1)) {
            // equal values (duplicated batch sizes): the lowest flat index i * Gs + s.  Winners with one
            // group of 64 and one count differ in the lane only, so the lowest lane has it; else a third minimum.
            where |= (int)((second >> lane) & 1ull) << 16;
            const int first_lane = __ffsll(winners) - 1;
            const int where0 = __builtin_amdgcn_readlane(where, first_lane);
            const unsigned long long same = __builtin_amdgcn_ballot_w64(where == where0);
            if ((winners & ~same) != 0) {
                const bool top = ((winners >> lane) & 1ull) != 0;
                const int flat = ((where >> 16) * kWave + lane) * Gs + (where & 0xFFFF);
                const int first = wave_min(top ? flat : 0x7FFFFFFF);
                winners &= __builtin_amdgcn_ballot_w64(flat == first);
            }
        }
    }
    const int wl = __ffsll(winners) - 1;
    const int wwhere = __builtin_amdgcn_readlane(where, wl);
    return Pick{((wwhere >> 16) | (int)((second >> wl) & 1ull)) * kWave + wl, wwhere & 0xFFFF};
}

// The same election for four (job, K, nodes) at once, one per row of 16 lanes, for small grids, where a sweep per
// wavefront spends more on its cross-lane steps than on the grid: every row of 16 lanes calls this with its own
// K (1 .. kTableK) and its own one_node (the same in all 16 lanes of a row; the job is the same for the whole
// wavefront), lane l of a row takes batch sizes l, l + 16, ..., and every lane of a row returns the row's
// result: (i << 16) | s of the feasible point with the smallest h, equal values to the lowest (i, s), or -1 when
// the row has no feasible point.  Per (K, batch size) the arithmetic is that of sweep_pick, instruction for
// instruction, so both elect the same point.
template <int CH, bool WHOLE>
__device__ __forceinline__ int sweep_pick_rows(const JobTables &tb, const RunSteps &X, const double *__restrict__ rs,
                                               int Gm, int Gs, int K, bool one_node, LdsDoubles near, bool has_near)
{
    const int l16 = lane_id() & 15;
    // Byte offsets inside one job's tables fit 32 bits (Gm <= 2^20, 2 * kTableK rows of 16 bytes per batch size): a
    // uniform base plus a 32-bit offset per lane, so that no address needs 64-bit vector arithmetic.
    const unsigned ca_row = (unsigned)((one_node ? kTableK : 0) + K - 1) * (unsigned)Gm * 16u;
    const unsigned s_row = (unsigned)(K - 1) * (unsigned)Gm * 4u;
    double kbest = __builtin_inf();   // smallest h seen by this lane
    int where = 0;                    // its (i << 16) | s
    const ScalarDoubles rsc = (ScalarDoubles)rs;
    for (int i0 = 0; i0 < Gm; i0 += 16) {
        const int i = i0 + l16;
        const bool feasible = WHOLE || i < Gm;       // WHOLE: Gm is a multiple of 64, so no lane runs past the grid
        const unsigned il = (unsigned)(feasible ? i : Gm - 1);
        const double tg = *(const double *)((const char *)tb.tg + 16u * il);
        const double2 car = *(const double2 *)((const char *)tb.ca + (ca_row + 16u * il));
        const double C = car.x, A0 = car.y;         // A0 = +inf when the batch size has no feasible count
        const int bounds = *(const int32_t *)((const char *)tb.srange + (s_row + 4u * il));
        const int s_lo = bounds & 0xFFFF, s_hi = bounds >> 16;
        const int s_star = scan_argmin<CH>(C, X, rsc, Gs, near, has_near);
        // convex w, feasible counts s_lo .. s_hi: the constrained argmin is the clamped one
        int s_c = s_star < s_hi ? s_star : s_hi;
        s_c = s_c > s_lo ? s_c : s_lo;
        double r_c, sd_c;
        if (has_near) {
            const Double2 rc = *(const Double2 __attribute__((address_space(3))) *)(near + 2 * s_c);
            r_c = rc.x;
            sd_c = rc.y;
        } else {
            r_c = rs[s_c];
            sd_c = (double)s_c;
        }
        const double w_c = px_fma(C, r_c, sd_c);
        const double key = px_fma(tg, w_c, A0);
        if (feasible && key < kbest) {
            kbest = key;
            where = (i << 16) | s_c;
        }
    }
    // Positive doubles order like their bit patterns: three unsigned minima over the row, the high words, the
    // low words among the lanes that hold the smallest high word, and (i, s) among the lanes that hold both.
    const unsigned hi = (unsigned)__double2hiint(kbest), lo = (unsigned)__double2loint(kbest);
    const unsigned hmin = row16_min(hi);
    const unsigned lmin = row16_min(hi == hmin ? lo : 0xFFFFFFFFu);
    const unsigned first = row16_min(hi == hmin && lo == lmin ? (unsigned)where : 0x7FFFFFFFu);
    return hmin >= 0x7FF00000u ? -1 : (int)first;             // every lane of the row still holds +inf: no point
}

template <int CH>
__device__ __forceinline__ Pick sweep_pick(const Job &q, const JobTables &tb, const double *__restrict__ rs,
                                           const double *__restrict__ rk, int Gm, int Gs, int K, int nodes)
{
    K = __builtin_amdgcn_readfirstlane(K);             // the same in every lane: scalar from here on
    nodes = __builtin_amdgcn_readfirstlane(nodes);
    if (K <= 0) return Pick{-1, -1};
    const RunSteps X = make_run_steps();
    if (tabled_row(K, nodes == 1, tb.k1)) return sweep_pick<CH, true>(q, tb, X, rs, rk, Gm, Gs, K, nodes);
    return sweep_pick<CH, false>(q, tb, X, rs, rk, Gm, Gs, K, nodes);
}

// Eq. 4 at grid point (i, s) in the paper's order of operations.  Arguments may differ
// from lane to lane.
__device__ __forceinline__ Best price_point(const Job &q, const JobTables &tb, int Gm, int K, bool one_node, int i, int s)
{
    if (i < 0) return Best{0.0, -1, -1};
    const int m = tb.m[i];
    const double tg = tb.tg[i].x;
    double last;
    if (tabled_row(K, one_node, tb.k1)) last = tb.lt[(unsigned)((one_node ? kTableK : 0) + K - 1) * (unsigned)Gm + (unsigned)i];
    else last = last_pass(sync_term(q, K, one_node), tg, tb.lntg[i]);
    return Best{goodput_point(q, (double)K * (double)m, tg, last, s), m, s};
}

// Sweep and price: every lane returns the same result.
template <int CH>
__device__ __forceinline__ Best sweep(const Job &q, const JobTables &tb, const double *__restrict__ rs,
                                      const double *__restrict__ rk, int Gm, int Gs, int K, int nodes)
{
    const Pick pick = sweep_pick<CH>(q, tb, rs, rk, Gm, Gs, K, nodes);
    return price_point(q, tb, Gm, K, nodes == 1, pick.i, pick.s);
}

__device__ __forceinline__ JobTables job_tables(const FitnessArgs &a, int j)
{
    const size_t o = (size_t)j * a.Gm;
    return JobTables{a.m_grid + o, a.tg + o, a.lntg + o, a.pu + o, a.qh5 + o, a.ql5 + o,
                     a.lt + (size_t)j * 2 * kTableK * a.Gm, a.ca + (size_t)j * 2 * kTableK * a.Gm,
                     a.srange + (size_t)j * kTableK * a.Gm, __builtin_amdgcn_readfirstlane(*a.k1)};
}

// ---- argmax by sampling total batch sizes (Sec. 4.3) -------------------------------
// The grid row of the job holds candidate total batch sizes M_i.  Lane l takes
// i = l, l+64, ...: s is the smallest accumulation count whose per-GPU batch
// m = ceil(M / (K (s+1))) stays within the memory bound, found with integer
// arithmetic; the point is then priced with Eq. 4 in the paper's order of operations
// (T_grad, its logarithm and the last pass of Eq. 10 are formed here, m is not on a grid).
// Gm evaluations per call instead of Gm * Gs.  Ties go to the lowest i.
__device__ __forceinline__ Best sweep_sampled(const Job &q, const int32_t *__restrict__ M_list, int Gm, int Gs, int K,
                                              int nodes)
{
    if (K <= 0) return Best{0.0, -1, -1};
    const int lane = lane_id();
    const double alpha_g = q.jp[(size_t)PX_ALPHA_G * q.J + q.j], beta_g = q.jp[(size_t)PX_BETA_G * q.J + q.j];
    const double M0 = q.jp[(size_t)PX_M0 * q.J + q.j], Mmax = q.jp[(size_t)PX_MMAX * q.J + q.j];
    const double m_mem_d = q.jp[(size_t)PX_M_MEM * q.J + q.j];
    if (!(m_mem_d >= 1.0 && m_mem_d <= 2147483647.0)) return Best{0.0, -1, -1};
    const long long per_pass = (long long)K * (long long)m_mem_d;     // examples one pass over K GPUs can hold
    const SyncTerm st = sync_term(q, K, nodes == 1);
    const double Kd = (double)K;

    double gbest = 0.0;
    int ibest = 0x7FFFFFFF, m_best = -1, s_best = -1;
    for (int i0 = 0; i0 < Gm; i0 += kWave) {
        const int i = i0 + lane;
        if (i >= Gm) continue;
        const long long M = M_list[i];
        if (M <= 0) continue;
        const long long s = (M + per_pass - 1) / per_pass - 1;
        if (s > (long long)(Gs - 1)) continue;
        const long long ks = (long long)K * (s + 1);
        const long long m = (M + ks - 1) / ks;                         // 1 <= m <= m_mem
        const double Km = Kd * (double)m;
        const double Mrun = Km * (double)(s + 1);
        if (Mrun < M0 || Mrun > Mmax) continue;
        const double tg = alpha_g + beta_g * (double)m;                // Eq. 8
        const double last = last_pass(st, tg, st.mode == 2 ? px_log(tg) : 0.0);
        const double g = goodput_point(q, Km, tg, last, (int)s);
        if (g > gbest) { gbest = g; ibest = i; m_best = (int)m; s_best = (int)s; }
    }
    return wave_argmax(gbest, ibest, m_best, s_best);
}

// ---- fp32 variant of the sweep --------------------------------------------------
// The same model with every parameter rounded to fp32 and all arithmetic of Eq. 4-11 in
// fp32 (powf for Eq. 10).  Each lane elects its best s with the rearranged form of the fp64
// sweep, evaluated in fp32, and prices the elected point with Eq. 4 in the plain form.  The
// feasibility interval M0 <= K m (s+1) <= M_max stays the exact integer test of the fp64
// path.  Ties go to the lowest flat index.

struct JobF32 {
    float alpha_g, beta_g, alpha_sl, beta_sl, alpha_sn, beta_sn, gamma, inv_gamma, phi, a;
};

__device__ __forceinline__ JobF32 load_job_f32(const double *__restrict__ jp, int J, int j)
{
    JobF32 q;
    q.alpha_g = (float)jp[(size_t)PX_ALPHA_G * J + j];
    q.beta_g = (float)jp[(size_t)PX_BETA_G * J + j];
    q.alpha_sl = (float)jp[(size_t)PX_ALPHA_SL * J + j];
    q.beta_sl = (float)jp[(size_t)PX_BETA_SL * J + j];
    q.alpha_sn = (float)jp[(size_t)PX_ALPHA_SN * J + j];
    q.beta_sn = (float)jp[(size_t)PX_BETA_SN * J + j];
    q.gamma = (float)jp[(size_t)PX_GAMMA * J + j];
    q.inv_gamma = 1.0f / q.gamma;
    q.phi = (float)jp[(size_t)PX_PHI * J + j];
    q.a = q.phi + (float)jp[(size_t)PX_M0 * J + j];
    return q;
}

__device__ __forceinline__ Best sweep_f32(const JobF32 &q, const JobTables &tb, const double *__restrict__ rk, int Gm,
                                          int Gs, int K, int nodes)
{
    Best out = {0.0, -1, -1};
    if (K <= 0) return out;
    const int lane = lane_id();
    const float Kf = (float)K;
    const double rK = K < kRecipTable ? rk[K] : 1.0 / (double)K;
    float ts = 0.0f;                                                          // Eq. 9
    if (K > 1) ts = (nodes == 1) ? q.alpha_sl + q.beta_sl * (float)(K - 2) : q.alpha_sn + q.beta_sn * (float)(K - 2);
    // Eq. 10 for K within the tables: the fp64 table of last_kernel, rounded to fp32 (two powf per batch size otherwise)
    const bool tabled = tabled_row(K, nodes == 1, tb.k1);
    const double *__restrict__ lrow = tb.lt + (unsigned)((nodes == 1 ? kTableK : 0) + (tabled ? K - 1 : 0)) * (unsigned)Gm;
    const float tsg = (!tabled && ts != 0.0f && q.gamma != 1.0f) ? powf(ts, q.gamma) : 0.0f;

    float gbest = -1.0f;
    int flat = 0x7FFFFFFF, m_best = -1, s_best = -1;
    for (int i0 = 0; i0 < Gm; i0 += kWave) {
        const int i = i0 + lane;
        if (i >= Gm) continue;
        const int m = tb.m[i];
        const float mf = (float)m;
        const float tg = q.alpha_g + q.beta_g * mf;                           // Eq. 8
        float last;                                                           // Eq. 10
        if (ts == 0.0f) last = tg;
        else if (q.gamma == 1.0f) last = tg + ts;
        else if (tabled) last = (float)lrow[i];
        else last = powf(powf(tg, q.gamma) + tsg, q.inv_gamma);
        const int s_lo = (int)(tb.ql5[i] * rK);
        int s_hi = (int)(tb.qh5[i] * rK) - 1;
        s_hi = s_hi < Gs - 1 ? s_hi : Gs - 1;
        // the lane's best s by the same rearrangement as the fp64 sweep, in fp32: argmax GOODPUT = argmin h,
        // h = (last + u tg) + s tg + (last - tg) u / (s + 1), u = phi / (K m); ties to the smaller s
        const float Km = Kf * mf;
        const float u = q.phi / Km;
        const float A0 = fmaf(u, tg, last), B0 = (last - tg) * u;
        float hbest = __builtin_inff();
        int sb = -1;
        for (int sI = s_lo; sI <= s_hi; ++sI) {
            const float h = fmaf(B0, __builtin_amdgcn_rcpf((float)(sI + 1)), fmaf((float)sI, tg, A0));
            if (h < hbest) { hbest = h; sb = sI; }
        }
        if (sb >= 0) {
            // Eq. 4 at the elected point, plain form
            const float M = Km * (float)(sb + 1);
            const float t_iter = (float)sb * tg + last;                      // Eq. 11
            const float g = (M / t_iter) * (q.a / (q.phi + M));              // Eq. 7 x Eq. 6
            if (g > gbest) { gbest = g; flat = i * Gs + sb; m_best = m; s_best = sb; }
        }
    }
    return wave_argmax((double)gbest, flat, m_best, s_best);
}

// ---- fp32 variant: the same scan-and-clamp sweep as the fp64 one ------------------------------
// For GPU counts within the tables.  Lane l owns batch sizes i = l, l + 64, ...; for each it scans
// w(s) = s + C / (s + 1) over all accumulation counts in chunks of 16, one v_fma_f32 per grid point
// (1/(s+1) from scalar registers, s from sixteen vector registers that hold 0 .. 15 for the whole
// kernel), one v_bfi_b32 that puts the position in the chunk into the low four mantissa bits, and one
// v_min3_f32 per two points: five instructions per two grid points.  The argmin over all counts is then
// put right between neighbours (the same exact test as in fp64: w(s+1) < w(s) exactly when
// C > (s+1)(s+2)), clamped to the feasible counts of (job, K, i) from the table, and h is formed there.
// The wave takes the smallest h (equal values: lowest flat index).  The elected point is priced with
// Eq. 4 in the plain form, in fp32 (price_point_f32).  T_grad, u and C are formed in fp32 from the
// parameters rounded to fp32; the last pass of Eq. 10 is the fp64 table rounded to fp32.
typedef const float __attribute__((address_space(4))) *ScalarFloats;
typedef const float __attribute__((address_space(3))) *LdsFloats;

struct RunStepsF32 {
    float x[16];
};

__device__ __forceinline__ RunStepsF32 make_run_steps_f32()
{
    RunStepsF32 X;
#pragma unroll
    for (int t = 0; t < 16; ++t) X.x[t] = (float)t;
    asm volatile("" : "+v"(X.x[0]), "+v"(X.x[1]), "+v"(X.x[2]), "+v"(X.x[3]), "+v"(X.x[4]), "+v"(X.x[5]), "+v"(X.x[6]), "+v"(X.x[7]));
    asm volatile("" : "+v"(X.x[8]), "+v"(X.x[9]), "+v"(X.x[10]), "+v"(X.x[11]), "+v"(X.x[12]), "+v"(X.x[13]), "+v"(X.x[14]), "+v"(X.x[15]));
    return X;
}

// Two grid points at positions B, B + 1 of a chunk: their values of w relative to the chunk's first count,
// tagged with their positions, folded into the running minimum.
template <int B>
__device__ __forceinline__ void scan_two_f32(float &kmin, float C, float r0, float r1, const RunStepsF32 &X)
{
    float w0, w1;
    int k0, k1;
    asm("v_fma_f32 %0, %1, %2, %3" : "=v"(w0) : "v"(C), "s"(r0), "v"(X.x[B]));
    asm("v_fma_f32 %0, %1, %2, %3" : "=v"(w1) : "v"(C), "s"(r1), "v"(X.x[B + 1]));
    asm("v_bfi_b32 %0, 15, %1, %2" : "=v"(k0) : "n"(B), "v"(__float_as_int(w0)));
    asm("v_bfi_b32 %0, 15, %1, %2" : "=v"(k1) : "n"(B + 1), "v"(__float_as_int(w1)));
    if constexpr (B == 0) asm("v_min_f32 %0, %1, %2" : "=v"(kmin) : "v"(__int_as_float(k0)), "v"(__int_as_float(k1)));
    else asm("v_min3_f32 %0, %0, %1, %2" : "+v"(kmin) : "v"(__int_as_float(k0)), "v"(__int_as_float(k1)));
}

template <int CH, int B = 0>
__device__ __forceinline__ void scan_chunk_f32(float &kmin, float C, ScalarFloats r, const RunStepsF32 &X)
{
    if constexpr (B < CH) {
        scan_two_f32<B>(kmin, C, r[B], r[B + 1], X);
        scan_chunk_f32<CH, B + 2>(kmin, C, r, X);
    }
}

// All 64 lanes call this with the same (job, 1 <= K <= kTableK, nodes); every lane returns the same result.
// rsf: 1/(s+1) in fp32, padded to a multiple of 32 counts; near: a copy of it in LDS when has_near.
template <int CH, bool WHOLE>
__device__ __forceinline__ Pick sweep_pick_f32(const JobF32 &q, const JobTables &tb, const RunStepsF32 &X,
                                               const float *__restrict__ rsf, int Gm, int Gs, int K, int nodes,
                                               LdsFloats near = nullptr, bool has_near = false)
{
    static_assert(CH == 8 || CH == 16, "positions of a chunk fit four tag bits");
    const int lane = lane_id();
    K = __builtin_amdgcn_readfirstlane(K);
    nodes = __builtin_amdgcn_readfirstlane(nodes);
    const bool one_node = nodes == 1;
    const float Kf = (float)K;
    float ts = 0.0f;                                                          // Eq. 9
    if (K > 1) ts = one_node ? q.alpha_sl + q.beta_sl * (float)(K - 2) : q.alpha_sn + q.beta_sn * (float)(K - 2);
    const int mode = ts == 0.0f ? 0 : (q.gamma == 1.0f ? 1 : 2);
    const double *__restrict__ lrow = tb.lt + (unsigned)((one_node ? kTableK : 0) + K - 1) * (unsigned)Gm;
    const int32_t *__restrict__ srow = tb.srange + (unsigned)(K - 1) * (unsigned)Gm;
    const ScalarFloats rsc = (ScalarFloats)rsf;

    float kbest = __builtin_inff();   // smallest h seen by this lane
    int where = 0;                    // its accumulation count | (index of its group of 64 batch sizes) << 16
    for (int i0 = 0; i0 < Gm; i0 += kWave) {
        const int i = i0 + lane;
        const bool active = WHOLE || i < Gm;
        const int il = active ? i : Gm - 1;
        const float mf = (float)tb.m[il];
        const float tg = q.alpha_g + q.beta_g * mf;                           // Eq. 8
        float last;                                                           // Eq. 10
        if (mode == 0) last = tg;
        else if (mode == 1) last = tg + ts;
        else last = (float)lrow[il];
        const float u = q.phi * __builtin_amdgcn_rcpf(Kf * mf);
        const float A0 = fmaf(u, tg, last);
        const float C = (last - tg) * u * __builtin_amdgcn_rcpf(tg);
        const int bounds = srow[il];
        const int s_lo = bounds & 0xFFFF, s_hi = bounds >> 16;
        const bool feasible = active && s_lo <= s_hi;
        // argmin of w over all counts: chunk by chunk, values relative to the chunk's first count
        float wmin;
        scan_chunk_f32<CH>(wmin, C, rsc, X);
        int s_star = __float_as_int(wmin) & 15;
        for (int s0 = CH; s0 < Gs; s0 += CH) {
            float w;
            scan_chunk_f32<CH>(w, C, rsc + s0, X);
            const float moved = w + (float)s0;                               // strictly smaller only: ties keep the smaller s
            if (moved < wmin) {
                wmin = moved;
                s_star = s0 + (__float_as_int(w) & 15);
            }
        }
        // neighbours in their exact order (the tags may have swapped two that agree to 2^-19)
        {
            const float sd = (float)s_star;
            const float t_lo = s_star > 0 ? fmaf(sd, sd, sd) : -1.0f, t_hi = fmaf(sd, sd, fmaf(3.0f, sd, 2.0f));
            s_star = C <= t_lo ? s_star - 1 : (C > t_hi ? s_star + 1 : s_star);
        }
        int s_c = s_star < s_hi ? s_star : s_hi;
        s_c = s_c > s_lo ? s_c : s_lo;
        const float r_c = has_near ? near[s_c] : rsf[s_c];
        const float key = fmaf(tg, fmaf(C, r_c, (float)s_c), A0);
        if (feasible && key < kbest) {
            kbest = key;
            where = s_c | ((i0 / kWave) << 16);
        }
    }
    // positive floats order like their bit patterns
    const unsigned bits = (unsigned)__float_as_int(kbest);
    const unsigned bmin = wave_min(bits);
    if (bmin >= 0x7F800000u) return Pick{-1, -1};               // every lane still holds +inf (or a NaN)
    unsigned long long winners = __builtin_amdgcn_ballot_w64(bits == bmin);
    if (winners & (winners - 1)) {
        // equal values: the lowest flat index i * Gs + s
        const bool top = ((winners >> lane) & 1ull) != 0;
        const int flat = ((where >> 16) * kWave + lane) * Gs + (where & 0xFFFF);
        const int first = wave_min(top ? flat : 0x7FFFFFFF);
        winners &= __builtin_amdgcn_ballot_w64(flat == first);
    }
    const int wl = __ffsll(winners) - 1;
    const int wwhere = __builtin_amdgcn_readlane(where, wl);
    return Pick{(wwhere >> 16) * kWave + wl, wwhere & 0xFFFF};
}

// Eq. 4 at grid point (i, s) in the plain form, in fp32, for a GPU count within the tables.  Arguments may
// differ from lane to lane.
__device__ __forceinline__ Best price_point_f32(const JobF32 &q, const JobTables &tb, int Gm, int K, bool one_node, int i, int s)
{
    if (i < 0) return Best{0.0, -1, -1};
    const int m = tb.m[i];
    const float mf = (float)m;
    const float tg = q.alpha_g + q.beta_g * mf;                               // Eq. 8
    float ts = 0.0f;                                                          // Eq. 9
    if (K > 1) ts = one_node ? q.alpha_sl + q.beta_sl * (float)(K - 2) : q.alpha_sn + q.beta_sn * (float)(K - 2);
    float last;                                                               // Eq. 10
    if (ts == 0.0f) last = tg;
    else if (q.gamma == 1.0f) last = tg + ts;
    else last = (float)tb.lt[(unsigned)((one_node ? kTableK : 0) + K - 1) * (unsigned)Gm + (unsigned)i];
    const float M = (float)K * mf * (float)(s + 1);
    const float t_iter = (float)s * tg + last;                                // Eq. 11
    const float g = (M / t_iter) * (q.a / (q.phi + M));                       // Eq. 7 x Eq. 6
    return Best{(double)g, m, s};
}

// The fp32 sweep of one (job, K, nodes) whatever K: scan and price within the tables, the plain loop beyond.
// Every lane returns the same result.
template <int CH>
__device__ __forceinline__ Best sweep_any_f32(const JobF32 &q, const JobTables &tb, const float *__restrict__ rsf,
                                              const double *__restrict__ rk, int Gm, int Gs, int K, int nodes)
{
    K = __builtin_amdgcn_readfirstlane(K);
    nodes = __builtin_amdgcn_readfirstlane(nodes);
    if (K <= 0) return Best{0.0, -1, -1};
    if (!tabled_row(K, nodes == 1, tb.k1)) return sweep_f32(q, tb, rk, Gm, Gs, K, nodes);
    const Pick pick = sweep_pick_f32<CH, false>(q, tb, make_run_steps_f32(), rsf, Gm, Gs, K, nodes);
    return price_point_f32(q, tb, Gm, K, nodes == 1, pick.i, pick.s);
}

// ---- per job -----------------------------------------------------------------

template <int CH, bool F32>
__global__ void __launch_bounds__(256) jobs_kernel(FitnessArgs a)
{
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int j = blockIdx.x * kWavesPerBlock + wave;
    if (j >= a.J) return;
    const int lane = lane_id();
    const Job q = load_job(a.job_params, a.J, j);
    const SyncParams y = load_sync(q);
    const double *__restrict__ jp = a.job_params;
    const double alpha_g = jp[(size_t)PX_ALPHA_G * a.J + j], beta_g = jp[(size_t)PX_BETA_G * a.J + j];
    const double M0 = jp[(size_t)PX_M0 * a.J + j], Mmax = jp[(size_t)PX_MMAX * a.J + j];
    const double w = jp[(size_t)PX_WEIGHT * a.J + j];
    const double T = jp[(size_t)PX_AGE_T * a.J + j];
    const double R = jp[(size_t)PX_RESTARTS_R * a.J + j];
    int st = 0;
    if (!(y.gamma >= 1.0 && y.gamma <= 10.0) || !(alpha_g >= 0.0) || !(beta_g >= 0.0) || !(y.alpha_sl >= 0.0) ||
        !(y.beta_sl >= 0.0) || !(y.alpha_sn >= 0.0) || !(y.beta_sn >= 0.0) || !(q.phi > 0.0) || !(M0 >= 1.0) ||
        !(Mmax >= M0) || !(w >= 0.0) || !(Mmax <= 4503599627370496.0) || !(alpha_g + beta_g > 0.0))
        st |= PX_ST_BAD_PARAM;
    if constexpr (CH == 0) {
        const double m_mem = jp[(size_t)PX_M_MEM * a.J + j];
        if (!(m_mem >= 1.0 && m_mem <= 2147483647.0)) st |= PX_ST_BAD_PARAM;
    }
    // re-allocation penalty factor of Sec. 4.2
    double factor = (T - R * a.delta) / (T + a.delta);
    if constexpr (F32) factor = (double)(((float)T - (float)R * (float)a.delta) / ((float)T + (float)a.delta));
    if (!(a.flags & PX_FLAG_NO_REALLOC_PENALTY) && !(T - R * a.delta > 0.0)) st |= PX_ST_BAD_RESTART;
    // does the job hold GPUs now?
    long long csum = 0;
    int neg = 0;
    for (int n = lane; n < a.N; n += kWave) {
        const int c = a.current_alloc[(size_t)j * a.N + n];
        csum += c;
        neg |= c < 0;
    }
    const long long total = wave_sum(csum);
    if (__ballot(neg) != 0) st |= PX_ST_NEG_ALLOC;
    // which 16-byte groups of the current row hold anything (rows that one 16-byte load per lane covers)
    unsigned long long groups = 0ull;
    if ((a.N & 3) == 0 && a.N <= 4 * kWave) {
        bool any = false;
        if (lane < (a.N >> 2)) {
            const int32_t *g = a.current_alloc + (size_t)j * a.N + 4 * lane;
            any = (g[0] | g[1] | g[2] | g[3]) != 0;
        }
        groups = __ballot(any);
    }
    // denominator of Eq. 15: the same sweep at the fair-share allocation
    Best fair;
    if constexpr (CH == 0)
        fair = sweep_sampled(q, a.m_grid + (size_t)j * a.Gm, a.Gm, a.Gs, a.fair_share[2 * j], a.fair_share[2 * j + 1]);
    else if constexpr (F32)
        fair = sweep_any_f32<CH>(load_job_f32(a.job_params, a.J, j), job_tables(a, j), a.rsf, a.rk, a.Gm, a.Gs,
                                 a.fair_share[2 * j], a.fair_share[2 * j + 1]);
    else
        fair = sweep<CH>(q, job_tables(a, j), a.rs, a.rk, a.Gm, a.Gs, a.fair_share[2 * j], a.fair_share[2 * j + 1]);
    if (!(fair.goodput > 0.0)) st |= PX_ST_ZERO_FAIR;
    if (lane == 0) {
        a.denom[j] = fair.goodput;
        a.factor[j] = (!(a.flags & PX_FLAG_NO_REALLOC_PENALTY) && total > 0) ? factor : 1.0;
        a.running[j] = total > 0;
        a.curmask[j] = groups;
        if (st) atomicOr(a.status, st);
    }
    if (j == 0 && lane < 16) a.zeros[lane] = 0;
}

// ---- memoised mode ---------------------------------------------------------------
// The goodput model sees an allocation row only through K and through whether the job
// sits on one node (Eq. 9), so the sweep of a pair equals the sweep of its (job, class, K).
// One wavefront per (job, class, K <= kTableK) runs the sweep once; the population pass
// then looks the result up (pairs_kernel with MEMO) and is bound by reading the
// population.  Rows with K > kTableK are swept in place.  Results are identical.
template <int CH, bool F32>
__global__ void __launch_bounds__(256) memo_kernel(FitnessArgs a)
{
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long row = (long long)blockIdx.x * kWavesPerBlock + wave;
    if (row >= (long long)a.J * 2 * kTableK) return;
    const int K = (int)(row % kTableK) + 1;
    const int nodes = ((row / kTableK) & 1) ? 1 : 2;
    const int j = (int)(row / (2 * kTableK));
    if (nodes == 1 && K > *a.k1) return;            // never looked up (tabled_row)
    Best best;
    if constexpr (CH == 0) best = sweep_sampled(load_job(a.job_params, a.J, j), a.m_grid + (size_t)j * a.Gm, a.Gm, a.Gs, K, nodes);
    else if constexpr (F32) best = sweep_any_f32<CH>(load_job_f32(a.job_params, a.J, j), job_tables(a, j), a.rsf, a.rk, a.Gm, a.Gs, K, nodes);
    else best = sweep<CH>(load_job(a.job_params, a.J, j), job_tables(a, j), a.rs, a.rk, a.Gm, a.Gs, K, nodes);
    if (lane_id() == 0) {
        MemoEntry e;
        e.goodput = best.goodput; e.m = best.m; e.s = best.s;
        a.memo[row] = e;
    }
}

// ---- per (candidate, job) ------------------------------------------------------
// Workgroup -> (job, group of candidates).  Workgroups are dealt to the eight XCDs
// round-robin, so the job index is derived from (blockIdx % 8) first: all workgroups
// of one job then run on one XCD and its tables stay in that XCD's L2.  Each of the
// four wavefronts walks cand_per_wave candidates of that job.

// ROW1: the host has checked that a row is at most 256 entries, a multiple of four, and that
// population and current_alloc are 16-byte aligned, so one 16-byte load per lane covers a row.
// WHOLE: the host has checked that Gm is a multiple of 64 (tabled sweeps then skip the test for the end of the grid).
// ROW4: ROW1 and a row is at most 64 entries, so one load of the wavefront covers the rows of four candidates
// (16 lanes each); cand_per_wave is at most 16.
// SEL: only the candidates listed in a.sel are evaluated (the children a search step has just formed); the
// wavefronts then walk positions of that list and look the candidate up where an address is formed.
// Eight wavefronts per SIMD (64 registers); the instances that sweep four candidates at a time (rows_at_a_time)
// take six (80 registers), which is what they need without spilling, and are no slower for it.
// Order of a wavefront's work (ROW1): request its first rows; fill the workgroup's table in LDS (entries formed
// in registers, so nothing waits for memory) and meet the other wavefronts; reduce the rows two at a time, and
// hand the registers of each finished pair to the rows of the next stretch of eight; then the sweeps of its
// candidates, one after the other; then prices and stores.  What a wavefront spends waiting at its start is
// time the vector ALU has one wavefront fewer to draw on, so memory is asked as early as the addresses are known.
// Between row pass and sweeps (grids of at most 128 batch sizes, whole groups of 64): the workgroup's 64 pairs
// share one job and mostly a handful of (placement class, GPU count) rows of its tables, so each pair votes for
// its row, the rows with two votes or more (four at most) are copied to LDS once, and the sweeps of those pairs
// read (C, A0), T_grad and the feasible range from there.  Three vector-memory loads per lane and group of 64
// batch sizes were what kept the texture addresser two thirds busy and the vector ALU waiting.
constexpr bool rows_at_a_time(int CH, bool F32, bool MEMO, bool ROW4) { return ROW4 && !F32 && !MEMO && CH != 0 && CH <= 16; }

// SEL = 2: per job, the candidates listed in a.dirty[j, 0 .. a.dirty_count[j]) (row inheritance: the rows of job j that a
// move or a repair of the search step has changed); workgroups beyond a job's list return at once.
template <int CH, bool F32, bool MEMO, bool ROW1, bool WHOLE = false, bool ROW4 = false, int SEL = 0>
__global__ void __launch_bounds__(256) __attribute__((amdgpu_waves_per_eu(rows_at_a_time(CH, F32, MEMO, ROW4) ? 6 : 8)))
pairs_kernel(FitnessArgs a)
{
    const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
    const int j = (slot / a.cand_groups) * 8 + xcd;
    const int group = slot % a.cand_groups;
    if (j >= a.J) return;
    // the number of candidates this job's workgroups share out among them
    int P_eff = SEL == 1 ? a.n_sel : a.P;
    if constexpr (SEL == 2) {
        P_eff = __builtin_amdgcn_readfirstlane(a.dirty_count[j]);
        if (group * a.cand_per_wave * kWavesPerBlock >= P_eff) return;
    }
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    // the reciprocals 1/(s+1) also in LDS when they fit: the clamped count of a lane reads its own entry
    // behind them U[t] = t (t+1), U[0] = -1: what decides the order of neighbouring counts (sweep_pick)
    // kStage: behind them the table rows most of the workgroup's pairs read (see kStageBase); stage_votes counts, per
    // (class, K), the pairs of the workgroup that read the row
    constexpr bool kStage = CH != 0 && !F32 && !MEMO && ROW1 && !ROW4 && WHOLE;
    __shared__ __align__(16) double r_lds[kNearU + kNearRecips + 8 + (kStage ? kStageDoubles : 0)];
    __shared__ int stage_votes[kStage ? 2 * kTableK : 1];
    // (only where the table of reciprocals and thresholds is in LDS as well: sweep_pick's staged path reads both)
    const bool stage_on = kStage && a.Gm <= kStageGm && a.gs_pad <= kNearRecips;
    bool has_near = false;
    // (the instances whose rows fit one 16-byte load per lane fill the table after they have requested their first rows)
    constexpr bool kRowsFirst = CH != 0 && ROW1;
    // every thread brings one entry, formed by the same division as the entry of a.rs (tables_kernel): no load, so
    // storing it waits for nothing that is on its way from memory
    static_assert(kNearRecips <= kWavesPerBlock * kWave, "one entry per thread");
    const bool near_fits = CH != 0 && !MEMO && a.gs_pad <= kNearRecips;
    const double near_d = 1.0 / (double)((int)threadIdx.x + 1);
    const float near_f = 1.0f / (float)((int)threadIdx.x + 1);
    auto fill_near = [&]() {
        if (near_fits) {
            const int t = threadIdx.x;
            if (t < a.gs_pad) {
                if constexpr (F32) {
                    ((float *)r_lds)[t] = near_f;
                } else {
                    r_lds[2 * t] = near_d;
                    r_lds[2 * t + 1] = (double)t;
                    for (int e = t; e < a.gs_pad + 8; e += a.gs_pad) {
                        const double ed = (double)e;
                        r_lds[kNearU + e] = e > 0 ? ed * (ed + 1.0) : -1.0;
                    }
                }
            }
        }
        if (stage_on && threadIdx.x < 2 * kTableK) stage_votes[threadIdx.x] = 0;
        if (near_fits || stage_on) __syncthreads();
        has_near = near_fits;
    };
    if constexpr (!kRowsFirst) fill_near();
    const Job q = load_job(a.job_params, a.J, j);
    JobF32 qf = {};
    if constexpr (F32) qf = load_job_f32(a.job_params, a.J, j);
    const JobTables tb = job_tables(a, j);
    const int32_t *__restrict__ cur = a.current_alloc + (size_t)j * a.N;
    const bool vec4 = ROW1 || ((a.N & 3) == 0 && (((uintptr_t)a.population | (uintptr_t)a.current_alloc) & 15) == 0);
    const int n4 = a.N >> 2;
    int4 cur0 = {0, 0, 0, 0};                         // the lane's share of the job's current row (its first 256 entries)
    if (vec4) cur0 = ((const int4 *)cur)[lane < n4 ? lane : n4 - 1];
    const int lane4 = lane < n4 ? lane : n4 - 1;      // ROW1: lanes past the end of the row load its last 16 bytes again
    const unsigned long long in_row = __ballot(lane < n4);
    constexpr bool kDeferred = CH != 0;               // the grid sweeps of both precisions (not the sampling argmax)
    constexpr int kPriced = -3;                       // a row beyond the tables whose result lane r already holds (see below)
    int d_K = 0, d_meta = 0, d_i = -1, d_s = -1;      // lane r: what candidate r of this wavefront needs at the end
    RunSteps X = {};
    RunStepsF32 XF = {};
    bool any_neg = false;

    // The wavefront's r-th candidate is c0 + kWavesPerBlock * r; its row of job j and its counters are reached
    // by stepping pointers.  With SEL that number is a position in the list, and lane r holds the candidate
    // listed there (-1 past the end of the list).
    const int c0 = group * a.cand_per_wave * kWavesPerBlock + wave;
    int d_c = -1;
    if constexpr (SEL != 0) {
        const int k = c0 + kWavesPerBlock * lane;
        if (lane < a.cand_per_wave && k < P_eff) d_c = SEL == 2 ? a.dirty[(size_t)j * a.n_sel + k] : a.sel[k];
    }
    const size_t row_step = (size_t)kWavesPerBlock * a.J * a.N;
    const int32_t *__restrict__ row = a.population + ((size_t)c0 * a.J + j) * a.N - row_step;
    unsigned long long *__restrict__ cp = a.colpack + (size_t)c0 * a.N - (size_t)kWavesPerBlock * a.N;
    // the row of job j of the wavefront's r-th candidate (SEL), and making that candidate the current one
    auto row_of = [&](int r) -> const int32_t * {
        return a.population + ((size_t)__builtin_amdgcn_readlane(d_c, r) * a.J + j) * a.N;
    };
    auto advance = [&](int r) {
        if constexpr (SEL != 0) {
            row = row_of(r);
            cp = a.colpack + (size_t)__builtin_amdgcn_readlane(d_c, r) * a.N;
        } else {
            row += row_step;
            cp += (size_t)kWavesPerBlock * a.N;
        }
    };

    // The row stage of the current candidate (see advance): row reduce and constraint counters.
    // ROW1 callers that have the row in registers already pass it as `have`; otherwise it is read here.  Callers
    // that have the row's sum already pass it as `K_have`, with `in_range` when they know that the row has no
    // negative entry.
    auto row_stage = [&](int &K_out, int &nodes_out, bool &changed_out, bool &neg_out, const int4 *have = nullptr,
                         const int *K_have = nullptr, int in_range = 0) {
        // row reduce: K = sum, nodes = #positive, changed = differs from the current row
        int ksum = 0, nodes = 0;
        bool changed = false, neg = false;
        int4 v0 = {0, 0, 0, 0};       // the lane's first four entries (the whole row when N <= 256)
        if constexpr (ROW1) {
            const int4 v = have ? *have : ((const int4 *)row)[lane4];
            v0 = v;
            if (!K_have) {
                const int part = (v.x + v.y) + (v.z + v.w);
                ksum = lane < n4 ? part : 0;
            }
            nodes = __popcll(__ballot(v.x > 0) & in_row) + __popcll(__ballot(v.y > 0) & in_row) +
                    __popcll(__ballot(v.z > 0) & in_row) + __popcll(__ballot(v.w > 0) & in_row);
            changed = ((__ballot(v.x != cur0.x) | __ballot(v.y != cur0.y) | __ballot(v.z != cur0.z) | __ballot(v.w != cur0.w)) & in_row) != 0;
            if (in_range == 0) neg = (__ballot((v.x | v.y | v.z | v.w) < 0) & in_row) != 0;
        } else if (vec4) {
            const int4 *__restrict__ row4 = (const int4 *)row;
            const int4 *__restrict__ cur4 = (const int4 *)cur;
            for (int n0 = 0; n0 < n4; n0 += kWave) {
                // lanes past the end of the row load its last 16 bytes again and are masked out of the ballots
                const int n = n0 + lane;
                const int nc = n < n4 ? n : n4 - 1;
                const int4 v = row4[nc];
                const int4 cv = n0 == 0 ? cur0 : cur4[nc];
                const unsigned long long valid = __ballot(n < n4);
                if (n0 == 0) v0 = v;
                const int part = (v.x + v.y) + (v.z + v.w);
                ksum += n < n4 ? part : 0;
                nodes += __popcll(__ballot(v.x > 0) & valid) + __popcll(__ballot(v.y > 0) & valid) +
                         __popcll(__ballot(v.z > 0) & valid) + __popcll(__ballot(v.w > 0) & valid);
                changed |= ((__ballot(v.x != cv.x) | __ballot(v.y != cv.y) | __ballot(v.z != cv.z) | __ballot(v.w != cv.w)) & valid) != 0;
                neg |= (__ballot((v.x | v.y | v.z | v.w) < 0) & valid) != 0;
            }
        } else {
            for (int n0 = 0; n0 < a.N; n0 += kWave) {
                const int n = n0 + lane;
                const int v = n < a.N ? row[n] : 0;
                const int cv = n < a.N ? cur[n] : 0;
                ksum += v;
                nodes += __popcll(__ballot(v > 0));
                changed |= __ballot(v != cv) != 0;
                neg |= __ballot(v < 0) != 0;
            }
        }
        const int K = K_have ? *K_have : wave_sum(ksum);

        // constraint check, part one: the row's non-zero entries (a job sits on few nodes) go to the
        // candidate's per-node counters; a multi-node job also counts once on each of its nodes.
        // One 64-bit integer atomic per entry: the result does not depend on the order of arrival.
        // (the flags of this stage are kept as integers in scalar registers: the compiler otherwise carries a
        // truth value across the branches as a lane mask that it rebuilds with two vector instructions)
        int need = __builtin_amdgcn_readfirstlane(a.need_constraints);
        asm volatile("" : "+s"(need));
        if (need != 0) {
            const unsigned long long one_job = nodes >= 2 ? kPackJob : 0ull;
            if ((ROW1 || (vec4 && a.N <= 4 * kWave)) && !neg) {
                // the row is still in registers and has no negative entry
                const int nb = lane * 4;
                if (lane < n4) {
                    if (v0.x > 0) atomicAdd(&cp[nb + 0], (unsigned long long)v0.x + one_job);
                    if (v0.y > 0) atomicAdd(&cp[nb + 1], (unsigned long long)v0.y + one_job);
                    if (v0.z > 0) atomicAdd(&cp[nb + 2], (unsigned long long)v0.z + one_job);
                    if (v0.w > 0) atomicAdd(&cp[nb + 3], (unsigned long long)v0.w + one_job);
                }
            } else {
                for (int n = lane; n < a.N; n += kWave) {
                    const int v = row[n];
                    if (v != 0) atomicAdd(&cp[n], (unsigned long long)(long long)v + (v > 0 ? one_job : 0ull));
                }
            }
        }
        K_out = K; nodes_out = nodes; changed_out = changed; neg_out = neg;
    };

    if constexpr (kDeferred) {
        // grid sweep (either precision), in two passes over the wavefront's candidates so that neither pass keeps the
        // other's addresses in scalar registers: first the row stage of every candidate (lane r keeps K and
        // nodes | changed of candidate r), then the sweeps, which elect a point per candidate; the points are
        // priced after the loop.
        int rows = a.cand_per_wave;
        if (c0 + kWavesPerBlock * (rows - 1) >= P_eff) rows = c0 < P_eff ? (P_eff - c0 + kWavesPerBlock - 1) / kWavesPerBlock : 0;
        if constexpr (ROW4) {
            // Lanes 16 g .. 16 g + 15 hold the row of candidate 4 b + g of the wavefront in batch b; all
            // batches are requested together.  Sums over a row are sums over 16 lanes (four DPP steps).
            static_assert(ROW1, "rows of 16-byte groups");
            const int g = lane >> 4, l16 = lane & 15;
            const bool in_row16 = l16 < n4;
            const int lane_off = in_row16 ? l16 : n4 - 1;
            const int4 *__restrict__ row1 = (const int4 *)(row + row_step) + lane_off;
            unsigned long long *__restrict__ cp1 = cp + (size_t)kWavesPerBlock * a.N + 4 * l16;
            const int4 curg = ((const int4 *)cur)[lane_off];
            constexpr int kBatches = kMaxCandPerWave / 4;
            int4 v[kBatches];
            int kb[kBatches] = {}, mb[kBatches] = {};
            int cb[kBatches] = {};           // SEL: the candidate whose row the lane holds in batch b
#pragma unroll
            for (int b = 0; b < kBatches; ++b) {
                if (4 * b < rows) {
                    const int r = 4 * b + g < rows ? 4 * b + g : rows - 1;             // the tail reads the last row again
                    if constexpr (SEL != 0) {
                        cb[b] = __builtin_amdgcn_ds_bpermute(r << 2, d_c);
                        v[b] = ((const int4 *)(a.population + ((size_t)cb[b] * a.J + j) * a.N))[lane_off];
                    } else {
                        v[b] = *(const int4 *)((const int32_t *)row1 + (size_t)r * row_step);
                    }
                }
            }
            fill_near();        // while the rows are on their way
#pragma unroll
            for (int b = 0; b < kBatches; ++b) {
                if (4 * b < rows) {
                    const int r = 4 * b + g;
                    const bool live = in_row16 && r < rows;
                    const int4 w = v[b];
                    const int part = (w.x + w.y) + (w.z + w.w);
                    const int positive = (w.x > 0 ? 1 : 0) + (w.y > 0 ? 1 : 0) + (w.z > 0 ? 1 : 0) + (w.w > 0 ? 1 : 0);
                    const int differs = ((w.x != curg.x) | (w.y != curg.y) | (w.z != curg.z) | (w.w != curg.w)) ? 1 : 0;
                    const int negative = ((w.x | w.y | w.z | w.w) < 0) ? 1 : 0;
                    // one word carries three small counts: positive entries (at most 64), lanes that differ, lanes with a negative entry
                    const int counts = row16_sum(live ? positive | (differs << 12) | (negative << 20) : 0);
                    const int K = row16_sum(live ? part : 0);
                    const int nodes = counts & 0xFFF;
                    kb[b] = K;
                    mb[b] = nodes | (((counts >> 12) & 0xFF) != 0 ? kMetaChanged : 0);
                    any_neg |= __ballot(live && (counts >> 20) != 0) != 0ull;
                    if (a.need_constraints && live) {
                        // every non-zero entry goes to the candidate's per-node counters (a negative one as it is)
                        const unsigned long long one_job = nodes >= 2 ? kPackJob : 0ull;
                        unsigned long long *__restrict__ to = SEL != 0 ? a.colpack + (size_t)cb[b] * a.N + 4 * l16
                                                                  : cp1 + (size_t)r * kWavesPerBlock * a.N;
                        if (w.x != 0) atomicAdd(&to[0], (unsigned long long)(long long)w.x + (w.x > 0 ? one_job : 0ull));
                        if (w.y != 0) atomicAdd(&to[1], (unsigned long long)(long long)w.y + (w.y > 0 ? one_job : 0ull));
                        if (w.z != 0) atomicAdd(&to[2], (unsigned long long)(long long)w.z + (w.z > 0 ? one_job : 0ull));
                        if (w.w != 0) atomicAdd(&to[3], (unsigned long long)(long long)w.w + (w.w > 0 ? one_job : 0ull));
                    }
                }
            }
            // lane r takes over what candidate r needs: from lane 16 (r mod 4) of batch r / 4
#pragma unroll
            for (int b = 0; b < kBatches; ++b) {
                const int from = ((lane & 3) * 16) << 2;
                const int K = __builtin_amdgcn_ds_bpermute(from, kb[b]), meta = __builtin_amdgcn_ds_bpermute(from, mb[b]);
                if ((lane >> 2) == b) {
                    d_K = K;
                    d_meta = meta;
                }
            }
        } else if constexpr (ROW1) {
            // eight rows are requested together: their latencies overlap.  The last eight come first: a stretch leaves
            // what its candidates need in lanes 0 .. 7, and the lanes move up by eight before the next stretch
            constexpr int kAhead = 8;
            static_assert(kMaxCandPerWave <= 2 * kAhead, "two stretches at most (the lanes move inside a row of 16)");
            const int r_last = (rows - 1) & ~(kAhead - 1);
            int at_row = -1;          // the candidate (of this wavefront) that `row` and `cp` point at
            int4 v[kAhead];
            const int32_t *__restrict__ row_first = row + row_step;       // the row of the wavefront's candidate 0 (SEL == 0)
            auto request = [&](int r, int4 &to) {
                const int ru = r < rows ? r : rows - 1;                   // the tail reads the last row again
                if constexpr (SEL != 0) to = ((const int4 *)row_of(ru))[lane4];
                else to = ((const int4 *)(row_first + (size_t)ru * row_step))[lane4];
            };
            // the rows of the first stretch are on their way while the workgroup fills its table in LDS
            if (r_last >= 0) {
#pragma unroll
                for (int u = 0; u < kAhead; ++u) request(r_last + u, v[u]);
            }
            fill_near();
            // One stretch; with hand_on the registers of its rows are handed on to the rows of the stretch below it, two
            // at a time.  (Written out once per stretch instead of as a loop, so that every wait names the loads it needs.)
            auto stretch = [&](int r0, auto hand_on) {
                if constexpr (SEL == 0) {
                    // advance() steps from one candidate to the next: start one before the stretch
                    const ptrdiff_t step = r0 - 1 - at_row;
                    row += step * (ptrdiff_t)row_step;
                    cp += step * (ptrdiff_t)kWavesPerBlock * a.N;
                    at_row = (r0 + kAhead < rows ? r0 + kAhead : rows) - 1;
                }
                // The sums of two rows come out of one reduction, 16 bits each, when every entry of both lies in
                // 0 .. 255 (a row of 256 such entries sums to less than 2^16), which the rows of any valid
                // population do; otherwise each row is summed on its own.
#pragma unroll
                for (int u = 0; u < kAhead; u += 2) {
                    if (r0 + u < rows) {
                        const int4 &va = v[u], &vb = v[u + 1];
                        int wide = (__ballot((unsigned)(((va.x | va.y) | (va.z | va.w)) | ((vb.x | vb.y) | (vb.z | vb.w))) > 255u) & in_row) != 0 ? 1 : 0;
                        wide = __builtin_amdgcn_readfirstlane(wide);
                        asm volatile("" : "+s"(wide));
                        const int part_a = lane < n4 ? (va.x + va.y) + (va.z + va.w) : 0;
                        const int part_b = lane < n4 ? (vb.x + vb.y) + (vb.z + vb.w) : 0;
                        int K2[2];
                        if (wide == 0) {
                            const int both = wave_sum(part_a + (part_b << 16));
                            K2[0] = both & 0xFFFF;
                            K2[1] = (int)((unsigned)both >> 16);
                        } else {
                            K2[0] = wave_sum(part_a);
                            K2[1] = wave_sum(part_b);
                        }
#pragma unroll
                        for (int e = 0; e < 2; ++e) {
                            if (r0 + u + e < rows) {
                                int K, nodes;
                                bool changed, neg;
                                advance(r0 + u + e);
                                row_stage(K, nodes, changed, neg, &v[u + e], &K2[e], wide ^ 1);
                                // lane r keeps what candidate r needs (see above)
                                d_K = write_lane8(d_K, K, u + e);
                                d_meta = write_lane8(d_meta, nodes | (changed ? kMetaChanged : 0), u + e);
                                any_neg |= neg;
                            }
                        }
                    }
                    // the rows of the next stretch take the registers this pair has left: they are on their way
                    // while the rest of this stretch is worked on
                    if constexpr (decltype(hand_on)::value) {
                        request(r0 - kAhead + u, v[u]);
                        request(r0 - kAhead + u + 1, v[u + 1]);
                    }
                }
            };
            if (r_last >= kAhead) {
                stretch(r_last, std::true_type());
                // (write_lane is an opaque statement: the two wait states a DPP read needs after a vector write of its
                // source are put here by hand, whatever the compiler schedules in between)
                asm volatile("s_nop 1" : "+v"(d_K), "+v"(d_meta));
                d_K = row16_up8(d_K);
                d_meta = row16_up8(d_meta);
            }
            if (r_last >= 0) stretch(0, std::false_type());
        } else {
            for (int r = 0; r < rows; ++r) {
                int K, nodes;
                bool changed, neg;
                advance(r);
                row_stage(K, nodes, changed, neg);
                if (lane == r) {
                    d_K = K;
                    d_meta = nodes | (changed ? kMetaChanged : 0);
                }
                any_neg |= neg;
            }
        }
        if constexpr (kStage) {
            if (stage_on) {
                // Which rows to stage: every pair of the workgroup votes for the row it will read, and every
                // wavefront takes, from the same counts (so all four agree), the rows with two votes or more: those
                // of the "one node" class first, fewer GPUs first, which is where allocations concentrate.  Lane r
                // then notes, in the register where the count elected for its candidate will go, where that
                // candidate's row is staged (-1: not staged).
                const int my_nodes = d_meta & ~kMetaChanged;
                const bool votes = lane < rows && d_K >= 1 && tabled_row(d_K, my_nodes == 1, tb.k1);
                const int my_row = (my_nodes == 1 ? kTableK : 0) + d_K - 1;
                if (votes) atomicAdd(&stage_votes[my_row], 1);
                __syncthreads();
                unsigned long long several = __ballot(stage_votes[lane] >= 2), one = __ballot(stage_votes[lane + kWave] >= 2);
                int staged[kStageRows];
                const int t = threadIdx.x;
                double2 ca_in[kStageRows];
                int range_in[kStageRows];
                double2 tg_in = {0.0, 0.0};
                if (t < a.Gm) tg_in = tb.tg[t];
#pragma unroll
                for (int e = 0; e < kStageRows; ++e) {
                    staged[e] = -1;
                    if (one != 0ull) {
                        staged[e] = kTableK + __builtin_ctzll(one);
                        one &= one - 1ull;
                    } else if (several != 0ull) {
                        staged[e] = __builtin_ctzll(several);
                        several &= several - 1ull;
                    }
                    if (staged[e] >= 0) {
                        // threads 0 .. Gm-1 bring the (C, A0) pairs of the row, threads Gm .. 2 Gm - 1 its feasible ranges
                        if (t < a.Gm) ca_in[e] = tb.ca[(size_t)staged[e] * a.Gm + t];
                        else if (t < 2 * a.Gm) range_in[e] = tb.srange[(size_t)(staged[e] & (kTableK - 1)) * a.Gm + (t - a.Gm)];
                        if (votes && my_row == staged[e]) d_s = kStageBase + 2 * kStageGm + e * kStageRowDoubles;
                    }
                }
                if (t < a.Gm) {
                    r_lds[kStageBase + 2 * t] = tg_in.x;
                    r_lds[kStageBase + 2 * t + 1] = tg_in.y;
                }
#pragma unroll
                for (int e = 0; e < kStageRows; ++e) {
                    if (staged[e] >= 0) {
                        double *row_lds = r_lds + kStageBase + 2 * kStageGm + e * kStageRowDoubles;
                        if (t < a.Gm) {
                            row_lds[2 * t] = ca_in[e].x;
                            row_lds[2 * t + 1] = ca_in[e].y;
                        } else if (t < 2 * a.Gm) {
                            ((int *)(row_lds + 2 * kStageGm))[t - a.Gm] = range_in[e];
                        }
                    }
                }
                __syncthreads();
            }
        }
        // after the row pass, whose rows in flight use the registers these occupy
        if constexpr (F32) XF = make_run_steps_f32();
        else X = make_run_steps();
        // Short rows come with small grids: there the sweeps go four candidates at a time, one per row of 16 lanes.
        constexpr bool kRows = rows_at_a_time(CH, F32, MEMO, ROW4);
        if constexpr (kRows) {
            const int g = lane >> 4;
            for (int b = 0; 4 * b < rows; ++b) {
                // lane r holds K and nodes of candidate r; this lane's row works on candidate 4 b + g
                const int r = 4 * b + g;
                const int K = __builtin_amdgcn_ds_bpermute(r << 2, d_K);
                const int nodes = __builtin_amdgcn_ds_bpermute(r << 2, d_meta) & ~kMetaChanged;
                const bool within = tabled_row(K, nodes == 1, tb.k1);
                const int K_in = (K < 1 || !within) ? 1 : K;
                // (this instance is launched only for grids whose tables of reciprocals and thresholds fit LDS)
                const int found = sweep_pick_rows<CH, WHOLE>(tb, X, a.rs, a.Gm, a.Gs, K_in, nodes == 1 && within, (LdsDoubles)r_lds, WHOLE || has_near);
                int pi = found < 0 ? -1 : found >> 16, ps = found < 0 ? -1 : found & 0xFFFF;
                if (K >= 1 && !within) {                     // rare: swept after the loop, outside the hot path
                    pi = kPending;
                    ps = -1;
                } else if (K < 1 || r >= rows) {
                    pi = -1;
                    ps = -1;
                }
                // lane 4 b + g' takes over what row g' has found
                const int from = ((lane & 3) * 16) << 2;
                const int ti = __builtin_amdgcn_ds_bpermute(from, pi), ts = __builtin_amdgcn_ds_bpermute(from, ps);
                if ((lane >> 2) == b) {
                    d_i = ti;
                    d_s = ts;
                }
            }
        }
        for (int r = 0; !kRows && r < rows; ++r) {
            const int K = __builtin_amdgcn_readlane(d_K, r);
            const int nodes = __builtin_amdgcn_readlane(d_meta, r) & ~kMetaChanged;
            Pick pick = {-1, -1};
            if (K >= 1 && !tabled_row(K, nodes == 1, tb.k1)) pick.i = kPending;   // rare: swept after the loop, outside the hot path
            else if (!MEMO && K >= 1) {
                if constexpr (F32) pick = sweep_pick_f32<CH, WHOLE>(qf, tb, XF, a.rsf, a.Gm, a.Gs, K, nodes, (LdsFloats)(const float *)r_lds, has_near);
                else pick = sweep_pick<CH, true, WHOLE>(q, tb, X, a.rs, a.rk, a.Gm, a.Gs, K, nodes, (LdsDoubles)r_lds, has_near,
                                                        kStage ? __builtin_amdgcn_readlane(d_s, r) : -1);
            }
            if (lane == r) {
                d_i = pick.i;
                d_s = pick.s;
            }
        }
    } else {
        // the sampling argmax: one candidate after the other, priced where it is swept
        for (int r = 0; r < a.cand_per_wave; ++r) {
            if (c0 + kWavesPerBlock * r >= P_eff) break;
            const int c = SEL != 0 ? __builtin_amdgcn_readlane(d_c, r) : c0 + kWavesPerBlock * r;
            int K, nodes;
            bool changed, neg;
            advance(r);
            row_stage(K, nodes, changed, neg);
            Best best;
            if (MEMO && K >= 1 && tabled_row(K, nodes == 1, tb.k1)) {
                const MemoEntry e = a.memo[((size_t)j * 2 + (nodes == 1 ? 1 : 0)) * kTableK + (K - 1)];
                best.goodput = e.goodput; best.m = e.m; best.s = e.s;
            } else {
                best = sweep_sampled(q, tb.m, a.Gm, a.Gs, K, nodes);
            }
            if (lane == 0) {
                const size_t pair = (size_t)c * a.J + j;
                a.G[pair] = best.goodput;
                a.meta[pair] = nodes | (changed ? kMetaChanged : 0);
                if (a.best_m) {
                    a.best_m[pair] = best.m;
                    a.best_s[pair] = best.s;
                }
                if (a.best_goodput) a.best_goodput[pair] = best.goodput;
                if (neg) atomicOr(a.status, PX_ST_NEG_ALLOC);
            }
        }
    }

    if constexpr (kDeferred) {
        // What follows needs pointers the loop above never touches (outputs, the tables of the
        // untabled path).  They are read from the kernel-argument segment again here, behind a
        // volatile statement, instead of occupying scalar registers throughout the loop.
        typedef const FitnessArgs __attribute__((address_space(4))) *KernelArgs;
        KernelArgs again = (KernelArgs)__builtin_amdgcn_kernarg_segment_ptr();
        asm volatile("" : "+s"(again));
        const FitnessArgs b = *(const FitnessArgs *)again;
        const Job qb = load_job(b.job_params, b.J, j);
        const JobTables tbb = job_tables(b, j);

        // rows with more GPUs than the tables cover: the whole wavefront sweeps and prices them one by one
        Best beyond = {0.0, -1, -1};
        unsigned long long pending = __ballot(d_i == kPending);
        while (pending) {
            const int l = __ffsll(pending) - 1;
            pending &= pending - 1;
            const int K = __builtin_amdgcn_readlane(d_K, l);
            const int nodes = __builtin_amdgcn_readlane(d_meta, l) & ~kMetaChanged;
            Best found;
            if constexpr (F32) {
                found = sweep_f32(qf, tbb, b.rk, b.Gm, b.Gs, K, nodes);
            } else {
                const Pick pick = sweep_pick<CH, false>(qb, tbb, X, b.rs, b.rk, b.Gm, b.Gs, K, nodes);
                found = price_point(qb, tbb, b.Gm, K, nodes == 1, pick.i, pick.s);
            }
            if (lane == l) {
                beyond = found;
                d_i = kPriced;
            }
        }
        // Lane l finishes the l-th candidate of this wavefront: the elected point is priced with
        // Eq. 4 in the paper's order of operations (or looked up in memoised mode) and stored.
        const int k = (group * b.cand_per_wave + lane) * kWavesPerBlock + wave;
        if (lane < b.cand_per_wave && k < (SEL == 2 ? P_eff : (SEL == 1 ? b.n_sel : b.P))) {
            const int c = SEL != 0 ? d_c : k;
            const size_t pair = (size_t)c * b.J + j;
            const int nodes = d_meta & ~kMetaChanged;
            Best best;
            if (MEMO && d_K >= 1 && tabled_row(d_K, nodes == 1, tbb.k1)) {
                const MemoEntry e = b.memo[((size_t)j * 2 + (nodes == 1 ? 1 : 0)) * kTableK + (d_K - 1)];
                best.goodput = e.goodput; best.m = e.m; best.s = e.s;
            } else if (d_i == kPriced) {
                best = beyond;
            } else if constexpr (F32) {
                best = price_point_f32(qf, tbb, b.Gm, d_K, nodes == 1, d_i, d_s);
            } else {
                best = price_point(qb, tbb, b.Gm, d_K, nodes == 1, d_i, d_s);
            }
            b.G[pair] = best.goodput;
            b.meta[pair] = d_meta;
            if (b.best_m) {
                b.best_m[pair] = best.m;
                b.best_s[pair] = best.s;
            }
            if (b.best_goodput) b.best_goodput[pair] = best.goodput;
        }
        if (any_neg && lane == 0) atomicOr(b.status, PX_ST_NEG_ALLOC);
    }
}

// ---- the argmax alone, for the consumers outside the search ----------------------------
// One wavefront per query (job, K, nodes): the same sweep and pricing as a (candidate, job) pair.
//   per_gpu mode   query (j, n), n = 0..max_nodes: column 0 is the job on one GPU, column n >= 1
//                  the job on n full nodes of gpus_per_node GPUs; the goodput is divided by the
//                  GPUs held (auto-scaling rule of Sec. 5.3.3)
//   tick mode      query j: the job at its current (K, nodes); its progress advances by
//                  goodput x (dt - restart delay if its allocation was changed) (Sec. 5.3)
struct QueryArgs {
    int mode;                       // 0 per_gpu, 1 tick
    int gpus_per_node, max_nodes;
    double *per_gpu;                // [J, max_nodes + 1]
    const int32_t *K, *nodes, *changed;
    const double *target;
    double dt, restart_delay;
    double *progress, *goodput;
    int32_t *finished;
};

template <int CH>
__global__ void __launch_bounds__(256) queries_kernel(FitnessArgs a, QueryArgs q)
{
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long id = (long long)blockIdx.x * kWavesPerBlock + wave;
    const int per_job = q.mode == 0 ? q.max_nodes + 1 : 1;
    if (id >= (long long)a.J * per_job) return;
    const int j = (int)(id / per_job), n = (int)(id % per_job);
    int K, nodes;
    if (q.mode == 0) {
        K = n == 0 ? 1 : n * q.gpus_per_node;
        nodes = n == 0 ? 1 : n;
    } else {
        K = q.K[j];
        nodes = q.nodes[j];
        if (!(q.progress[j] < q.target[j])) K = 0;              // a finished job is left as it is
    }
    K = __builtin_amdgcn_readfirstlane(K);             // one query per wavefront: the same in every lane
    nodes = __builtin_amdgcn_readfirstlane(nodes);
    Best best = {0.0, -1, -1};
    if (K > 0) best = sweep<CH>(load_job(a.job_params, a.J, j), job_tables(a, j), a.rs, a.rk, a.Gm, a.Gs, K, nodes);
    if (lane_id() != 0) return;
    if (q.mode == 0) {
        q.per_gpu[id] = best.goodput / (double)K;
    } else {
        const double before = q.progress[j];
        const double run = q.dt - (q.changed[j] ? q.restart_delay : 0.0);
        const double after = (K > 0 && run > 0.0) ? before + best.goodput * run : before;
        q.goodput[j] = best.goodput;
        q.progress[j] = after;
        q.finished[j] = after >= q.target[j];
    }
}

// Sec. 5.3.3: a job scales up when its goodput per GPU exceeds U of the ideal (one GPU, column 0), to the
// node count reached by adding nodes while the next count still predicts at least L of the ideal per GPU.
__global__ void __launch_bounds__(256) autoscale_kernel(int J, int max_nodes, const double *__restrict__ per_gpu,
                                                       const int32_t *__restrict__ nodes_now, double U, double L,
                                                       int32_t *__restrict__ nodes_new)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= J) return;
    const double *__restrict__ row = per_gpu + (size_t)j * (max_nodes + 1);
    int n = nodes_now[j];
    if (n >= 1 && n <= max_nodes && row[n] > U * row[0]) {
        while (n < max_nodes && row[n + 1] >= L * row[0]) ++n;
    }
    nodes_new[j] = n;
}

// ---- per candidate -------------------------------------------------------------

constexpr int kCandThreads = 256;

__device__ __forceinline__ double pmean_term(double s, double w, double p)
{
    if (p == 0.0) return w * log(s);      // log(0) = -inf
    if (p == 1.0) return w * s;
    if (p == -1.0) return w * (1.0 / s);  // 1/0 = +inf, as pow(0, -1)
    return w * pow(s, p);                 // pow(0, p<0) = +inf
}

__device__ __forceinline__ float pmean_term(float s, float w, float p)
{
    if (p == 0.0f) return w * logf(s);
    return w * powf(s, p);
}

__device__ __forceinline__ double pmean_finish(double mean, double p)
{
    if (p == 0.0) return exp(mean);
    if (p == 1.0) return mean;
    if (p == -1.0) return 1.0 / mean;
    return pow(mean, 1.0 / p);
}
__device__ __forceinline__ float pmean_finish(float mean, float p) { return p == 0.0f ? expf(mean) : powf(mean, 1.0f / p); }

// REAL = double, or float for the fp32 variant (SPEEDUP, the penalty and the mean are then formed in fp32).
template <typename REAL>
__global__ void __launch_bounds__(kCandThreads) candidates_kernel(FitnessArgs a)
{
    __shared__ REAL red_acc[kCandThreads];
    __shared__ REAL red_w[kCandThreads];
    __shared__ long long red_v[kCandThreads];
    const int c = a.sel ? a.sel[blockIdx.x] : (int)blockIdx.x;
    const int t = threadIdx.x;
    const double *__restrict__ G = a.G + (size_t)c * a.J;
    const int32_t *__restrict__ meta = a.meta + (size_t)c * a.J;
    const double *__restrict__ wt = a.job_params + (size_t)PX_WEIGHT * a.J;

    // SPEEDUP (Eq. 15) with the re-allocation penalty, then the generalized mean (Eq. 14):
    // each thread sums its jobs in ascending order, then a fixed tree
    REAL acc = 0, wsum = 0;
    const REAL p = (REAL)a.p;
    for (int j = t; j < a.J; j += kCandThreads) {
        const REAL d = (REAL)a.denom[j];
        REAL s_j = d > 0 ? (REAL)G[j] / d : (REAL)0;
        if (meta[j] & kMetaChanged) s_j = s_j * (REAL)a.factor[j];
        if (a.speedup) a.speedup[(size_t)c * a.J + j] = (double)s_j;
        acc += pmean_term(s_j, (REAL)wt[j], p);
        wsum += (REAL)wt[j];
    }
    red_acc[t] = acc;
    red_w[t] = wsum;

    // constraint check, part two: per node, multi-node jobs beyond the first and GPUs beyond capacity
    long long v = 0;
    if (a.need_constraints) {
        // the counters are left at zero for the next call on this workspace (see launch_fitness)
        unsigned long long *__restrict__ cp = a.colpack + (size_t)c * a.N;
        for (int n = t; n < a.N; n += kCandThreads) {
            const long long x = (long long)cp[n];
            cp[n] = 0ull;
            const long long asked = (x << 24) >> 24;              // low 40 bits, sign-extended
            const long long distributed = (x - asked) >> 40;
            if (distributed > 1) v += distributed - 1;
            const long long over = asked - (long long)a.node_capacity[n];
            if (over > 0) v += over;
        }
    }
    red_v[t] = v;
    __syncthreads();
    for (int half = kCandThreads / 2; half > 0; half >>= 1) {
        if (t < half) {
            red_acc[t] += red_acc[t + half];
            red_w[t] += red_w[t + half];
            red_v[t] += red_v[t + half];
        }
        __syncthreads();
    }
    if (t == 0) {
        const REAL mean = red_acc[0] / red_w[0];
        double f = (double)pmean_finish(mean, (REAL)a.p);
        const long long V = red_v[0];
        if (a.violations) a.violations[c] = (int32_t)(V > 0x7FFFFFFF ? 0x7FFFFFFF : V);
        if (V > 0 && !(a.flags & PX_FLAG_NO_CONSTRAINT_CHECK)) f = -(double)V;
        a.fitness[c] = f;
    }
}

// ---- row inheritance (pollux_generation with PX_GA_INHERIT_ROWS) ----------------------------------
// The search step has left, per child it formed and per job, the candidate whose row the child holds unchanged
// (a survivor: its results are in place), or -1.  Eq. 13, the re-allocation flag and everything else the fitness
// takes from a row depend on the row, the job and the current allocation only, so an unchanged row takes over the
// results of its source.  The rows a move or a repair has changed are listed per job (a.dirty[j, ...], counted in
// a.dirty_count[j]) for pairs_kernel with SEL = 2, which treats them like any other (candidate, job) pair, per-node
// counters included.  A child the step has flagged (a.odd: it may hold a negative entry or violate a constraint)
// lists all its rows, so its counters come out complete; of every other child only some rows reach the counters,
// and a part of a matrix that satisfies both constraints (which such a child does by construction) satisfies
// them too, so its violation count is the zero it has to be.  One workgroup per listed child; candidates_kernel
// follows as usual.
__global__ void __launch_bounds__(256) inherit_kernel(FitnessArgs a)
{
    const int k = blockIdx.x;
    const int slot = a.sel[k];
    const bool odd = a.odd[k] != 0;
    const int32_t *__restrict__ src = a.src_row + (size_t)k * a.J;
    // four jobs per thread and pass: the sources first, then all the reads that depend on them, then the stores
    constexpr int kJobs = 4;
    for (int j0 = threadIdx.x; j0 < a.J; j0 += kJobs * 256) {
        int s[kJobs];
#pragma unroll
        for (int u = 0; u < kJobs; ++u) {
            const int j = j0 + u * 256;
            s[u] = (j < a.J && !odd) ? src[j] : -1;
        }
        double g[kJobs], bg[kJobs];
        int32_t mt[kJobs], bm[kJobs], bs[kJobs];
#pragma unroll
        for (int u = 0; u < kJobs; ++u) {
            const size_t from = (size_t)(s[u] >= 0 ? s[u] : slot) * a.J + (j0 + u * 256 < a.J ? j0 + u * 256 : 0);
            g[u] = a.G[from];
            mt[u] = a.meta[from];
            bm[u] = a.best_m ? a.best_m[from] : 0;
            bs[u] = a.best_m ? a.best_s[from] : 0;
            bg[u] = a.best_goodput ? a.best_goodput[from] : 0.0;
        }
#pragma unroll
        for (int u = 0; u < kJobs; ++u) {
            const int j = j0 + u * 256;
            if (j >= a.J) continue;
            const size_t to = (size_t)slot * a.J + j;
            if (s[u] >= 0) {
                a.G[to] = g[u];
                a.meta[to] = mt[u];
                if (a.best_m) {
                    a.best_m[to] = bm[u];
                    a.best_s[to] = bs[u];
                }
                if (a.best_goodput) a.best_goodput[to] = bg[u];
            } else {
                a.dirty[(size_t)j * a.n_sel + atomicAdd(&a.dirty_count[j], 1)] = slot;
            }
        }
    }
}

// ---- memoised mode, one workgroup per candidate ---------------------------------------------------
// With the sweeps looked up a candidate costs the reading of its matrix and little else, so one workgroup
// takes the whole candidate: it walks the matrix in memory order (four wavefronts, 64 consecutive rows each
// per round of 256 jobs, four rows and the matching rows of the current allocation requested at a time, the
// next four before the current ones are worked on, from one round straight into the next), keeps the per-node
// counters of the constraint check in LDS (integer atomics: order-independent) and K, nodes and the changed flag
// of every row in LDS as well.  After up to 1024 jobs the workgroup stops reading, and thread t finishes the
// pairs of jobs t, t + 256, ... of those: looks the sweep's result up, forms SPEEDUP (Eq. 15) with the penalty
// and its term of the generalized mean (Eq. 14).  (Finishing per round instead, between the requests, left the
// memory system idle a tenth of the time.)  The terms are summed exactly as candidates_kernel sums them (thread
// t over its jobs in ascending order, then the same tree), so the fitness is bit-identical to the plain mode's.
// Nothing but the results leaves the chip.  For rows of 16-byte groups of at most 256 nodes, fp64, grid sweeps
// (not the sampling argmax).
// BEYOND = false: the instance for the common case.  A candidate with a row of more GPUs than the memo table
// covers is left alone and flagged in a.redo[c]; the instance with BEYOND = true is launched after it, returns at
// once for the candidates that are done and treats the flagged ones in full, such rows swept by their wavefront.
// Split because the sweep costs the kernel twice the registers of everything else in it.
constexpr int kMemoChunkJobs = 4 * kCandThreads;    // jobs between two finishing steps

// PAIRS: the goodput and the node count of every pair are also left in the workspace (PX_FLAG_PAIR_RESULTS).
template <int CH, bool BEYOND, bool PAIRS>
__global__ void __launch_bounds__(kCandThreads) memo_candidates_kernel(FitnessArgs a)
{
    static_assert(kCandThreads == 4 * kWave, "thread t of the workgroup is lane t % 64 of wavefront t / 64");
    constexpr int kAhead = 4;
    static_assert(kWave % (2 * kAhead) == 0, "a pass of the request loop never straddles two rounds");
    __shared__ unsigned long long node_lds[4 * kWave];       // per node: GPUs asked + multi-node jobs << 40, as colpack
    __shared__ int2 row_lds[kMemoChunkJobs];                  // per job of the chunk: K, nodes | changed flag
    __shared__ MemoEntry beyond_lds[BEYOND ? kMemoChunkJobs : 1];   // per job of the chunk with K beyond the table: its sweep
    __shared__ double red_acc[kCandThreads];
    __shared__ double red_w[kCandThreads];
    __shared__ long long red_v[kCandThreads];
    __shared__ int found_beyond;
    const int c = a.sel ? a.sel[blockIdx.x] : (int)blockIdx.x;
    if constexpr (BEYOND) {
        if (!a.redo[c]) return;
    }
    const int t = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int lane = lane_id();
    const int n4 = a.N >> 2;
    const int lane4 = lane < n4 ? lane : n4 - 1;          // lanes past the end of a row load its last 16 bytes again
    const unsigned long long in_row = __ballot(lane < n4);
    const double *__restrict__ wt = a.job_params + (size_t)PX_WEIGHT * a.J;
    const int k1 = __builtin_amdgcn_readfirstlane(*a.k1);
    node_lds[t] = 0ull;
    if (t == 0) found_beyond = 0;
    __syncthreads();

    double acc = 0.0, wsum = 0.0;
    bool any_neg = false;
    for (int jc = 0; jc < a.J; jc += kMemoChunkJobs) {
        const int chunk_jobs = a.J - jc < kMemoChunkJobs ? a.J - jc : kMemoChunkJobs;
        // Row q of this wavefront in the chunk is job  jc + (q / 64) * 256 + 64 * wave + q % 64  (position in the
        // chunk: the same without jc); the wavefront has `rows` of them.
        int tail = chunk_jobs % kCandThreads - kWave * wave;
        tail = tail < 0 ? 0 : (tail > kWave ? kWave : tail);
        const int rows = kWave * (chunk_jobs / kCandThreads) + tail;
        auto place = [&](int q) { return (q >> 6) * kCandThreads + kWave * wave + (q & (kWave - 1)); };
        if (rows > 0) {
            const int4 *__restrict__ rowp = (const int4 *)(a.population + ((size_t)c * a.J + jc) * a.N) + lane4;
            const int4 *__restrict__ curp = (const int4 *)(a.current_alloc + (size_t)jc * a.N) + lane4;
            auto request = [&](int q0, int4 (&v)[kAhead]) {
#pragma unroll
                for (int u = 0; u < kAhead; ++u) {
                    const int q = q0 + u < rows ? q0 + u : rows - 1;               // the tail reads the last row again
                    v[u] = rowp[(size_t)place(q) * n4];
                }
            };
            // The rows of the current allocation come from L2 (shared by all candidates), and only the lanes whose
            // 16-byte group of the current row holds anything read it (a.curmask, a scalar per row: a job sits on few
            // nodes, so that is a lane or two); all other lanes read one block of zeros, which is what the current
            // row holds there: a few cache lines per row through the vector cache instead of 1 KB.  Every lane
            // loads either way, so the number of loads in flight is the same on every path and the waits can be
            // exact.  The rows are requested when their batch is about to be worked on, not a batch ahead, which
            // saves the registers of a second buffer, but BEFORE the next batch of the population is requested:
            // loads complete in order, so waiting for them then leaves that next batch in flight.
            // (the masks through the scalar cache: a vector load would make every use wait for all loads in flight)
            typedef const unsigned long long __attribute__((address_space(4))) *ScalarMasks;
            const ScalarMasks maskp = (ScalarMasks)a.curmask + jc;
            const int4 *__restrict__ zerop = (const int4 *)a.zeros;
            auto request_current = [&](int q0, int4 (&cv)[kAhead]) {
#pragma unroll
                for (int u = 0; u < kAhead; ++u) {
                    const int at = place(q0 + u < rows ? q0 + u : rows - 1);
                    cv[u] = *(((maskp[at] >> lane) & 1ull) ? curp + (size_t)at * n4 : zerop);
                }
            };
            int d_K = 0, d_meta = 0;                        // lane r: K and nodes | changed of row q with q % 64 = r
            auto work = [&](int q0, const int4 (&v)[kAhead], const int4 (&cv)[kAhead]) {
#pragma unroll
                for (int u = 0; u < kAhead; ++u) {
                    if (q0 + u < rows) {
                        const int4 w = v[u], was = cv[u];
                        const int part = (w.x + w.y) + (w.z + w.w);
                        const int K = wave_sum(lane < n4 ? part : 0);
                        const int nodes = __popcll(__ballot(w.x > 0) & in_row) + __popcll(__ballot(w.y > 0) & in_row) +
                                          __popcll(__ballot(w.z > 0) & in_row) + __popcll(__ballot(w.w > 0) & in_row);
                        const bool changed = ((__ballot(w.x != was.x) | __ballot(w.y != was.y) | __ballot(w.z != was.z) | __ballot(w.w != was.w)) & in_row) != 0;
                        any_neg |= (__ballot((w.x | w.y | w.z | w.w) < 0) & in_row) != 0;
                        if (a.need_constraints && lane < n4 && (w.x | w.y | w.z | w.w) != 0) {
                            // The few lanes that hold a non-zero entry (a job sits on few nodes) add their four
                            // entries to the per-node counters, zeros included (a negative entry as it is): one
                            // branch per row instead of one per entry.
                            const unsigned long long one_job = nodes >= 2 ? kPackJob : 0ull;
                            unsigned long long *to = node_lds + 4 * lane;
                            atomicAdd(&to[0], (unsigned long long)(long long)w.x + (w.x > 0 ? one_job : 0ull));
                            atomicAdd(&to[1], (unsigned long long)(long long)w.y + (w.y > 0 ? one_job : 0ull));
                            atomicAdd(&to[2], (unsigned long long)(long long)w.z + (w.z > 0 ? one_job : 0ull));
                            atomicAdd(&to[3], (unsigned long long)(long long)w.w + (w.w > 0 ? one_job : 0ull));
                        }
                        if (lane == ((q0 + u) & (kWave - 1))) {
                            d_K = K;
                            d_meta = nodes | (changed ? kMetaChanged : 0);
                        }
                    }
                }
            };
            // Two buffers of kAhead rows: requests are in flight all the time.  A request past the end of the
            // wavefront's rows reads its last row again (nothing works on it), so that every pass through the
            // loop issues the same loads in the same order and each wait leaves exactly the next batch in flight.
            int4 v0[kAhead], v1[kAhead], cv[kAhead];
            request(0, v0);
            // (the fences keep the compiler from issuing the requests in another order)
            auto fence = [] {
                asm volatile("" ::: "memory");
                __builtin_amdgcn_sched_barrier(0);
            };
            for (int q0 = 0; q0 < rows; q0 += 2 * kAhead) {
                request_current(q0, cv);
                fence();
                request(q0 + kAhead, v1);
                fence();
                work(q0, v0, cv);
                fence();
                request_current(q0 + kAhead, cv);
                fence();
                request(q0 + 2 * kAhead, v0);
                fence();
                work(q0 + kAhead, v1, cv);
                fence();
                // a round of 64 rows (or the last, shorter one) is complete: lane r puts its row's figures away
                const int next = q0 + 2 * kAhead;
                if ((next & (kWave - 1)) == 0 || next >= rows) {
                    const int first = q0 & ~(kWave - 1);
                    const int in_round = rows - first < kWave ? rows - first : kWave;
                    const int at = place(first) + lane;
                    if (lane < in_round) row_lds[at] = make_int2(d_K, d_meta);
                    // rows beyond the memo table: swept and priced by the whole wavefront (BEYOND), or the candidate
                    // is left to the instance that can
                    unsigned long long pending = __ballot(lane < in_round && !tabled_row(d_K, (d_meta & ~kMetaChanged) == 1, k1));
                    if constexpr (BEYOND) {
                        while (pending) {
                            const int l = __ffsll(pending) - 1;
                            pending &= pending - 1;
                            const int K = __builtin_amdgcn_readlane(d_K, l);
                            const int nodes = __builtin_amdgcn_readlane(d_meta, l) & ~kMetaChanged;
                            const int j = jc + place(first) + l;
                            const Best b = sweep<CH>(load_job(a.job_params, a.J, j), job_tables(a, j), a.rs, a.rk, a.Gm, a.Gs, K, nodes);
                            if (lane == l) {
                                MemoEntry e;
                                e.goodput = b.goodput; e.m = b.m; e.s = b.s;
                                beyond_lds[at] = e;
                            }
                        }
                    } else if (pending) {
                        if (lane == 0) found_beyond = 1;
                    }
                }
            }
        }
        __syncthreads();                                    // the chunk's rows are all put away
        if constexpr (!BEYOND) {
            // (the outputs written so far for a flagged candidate are written again, in full, by the other instance)
            if (found_beyond) {
                if (t == 0) a.redo[c] = 1;
                return;
            }
        }
        // thread t finishes the pairs of jobs jc + t, jc + t + 256, ...
        for (int at = t; at < chunk_jobs; at += kCandThreads) {
            const int j = jc + at;
            const size_t pair = (size_t)c * a.J + j;
            const int2 row = row_lds[at];
            const int d_K = row.x, d_meta = row.y;
            const int nodes = d_meta & ~kMetaChanged;
            Best best = {0.0, -1, -1};
            if (d_K >= 1 && tabled_row(d_K, nodes == 1, k1)) {
                const MemoEntry e = a.memo[((size_t)j * 2 + (nodes == 1 ? 1 : 0)) * kTableK + (d_K - 1)];
                best.goodput = e.goodput; best.m = e.m; best.s = e.s;
            } else if (BEYOND && d_K >= 1) {
                const MemoEntry e = beyond_lds[at];
                best.goodput = e.goodput; best.m = e.m; best.s = e.s;
            }
            if (a.best_m) {
                a.best_m[pair] = best.m;
                a.best_s[pair] = best.s;
            }
            if (a.best_goodput) a.best_goodput[pair] = best.goodput;
            if constexpr (PAIRS) {
                // what a later generation that inherits rows reads of this pair
                a.G[pair] = best.goodput;
                a.meta[pair] = d_meta;
            }
            // SPEEDUP (Eq. 15) with the re-allocation penalty, and the job's term of Eq. 14
            const double d = a.denom[j];
            double s_j = d > 0 ? best.goodput / d : 0.0;
            if (d_meta & kMetaChanged) s_j = s_j * a.factor[j];
            if (a.speedup) a.speedup[pair] = s_j;
            acc += pmean_term(s_j, wt[j], a.p);
            wsum += wt[j];
        }
        __syncthreads();                                    // before the next chunk's rows take their places
    }
    red_acc[t] = acc;
    red_w[t] = wsum;
    if constexpr (!BEYOND) {
        if (t == 0) a.redo[c] = 0;
    }
    if (__ballot(any_neg) != 0ull && lane == 0) atomicOr(a.status, PX_ST_NEG_ALLOC);

    // constraint check: per node, multi-node jobs beyond the first and GPUs beyond capacity
    long long v = 0;
    if (a.need_constraints && t < a.N) {
        const long long x = (long long)node_lds[t];
        const long long asked = (x << 24) >> 24;              // low 40 bits, sign-extended
        const long long distributed = (x - asked) >> 40;
        if (distributed > 1) v += distributed - 1;
        const long long over = asked - (long long)a.node_capacity[t];
        if (over > 0) v += over;
    }
    red_v[t] = v;
    __syncthreads();
    for (int half = kCandThreads / 2; half > 0; half >>= 1) {
        if (t < half) {
            red_acc[t] += red_acc[t + half];
            red_w[t] += red_w[t + half];
            red_v[t] += red_v[t + half];
        }
        __syncthreads();
    }
    if (t == 0) {
        const double mean = red_acc[0] / red_w[0];
        double f = pmean_finish(mean, a.p);
        const long long V = red_v[0];
        if (a.violations) a.violations[c] = (int32_t)(V > 0x7FFFFFFF ? 0x7FFFFFFF : V);
        if (V > 0 && !(a.flags & PX_FLAG_NO_CONSTRAINT_CHECK)) f = -(double)V;
        a.fitness[c] = f;
    }
}

}  // namespace px

// ---- host side -----------------------------------------------------------------

namespace px {

// The job-level part of the arguments: dimensions, inputs that describe the jobs, workspace sections.
static FitnessArgs job_level_args(const pollux_dims *d, const double *job_params, const int32_t *m_grid, void *workspace)
{
    const WorkspaceLayout L = workspace_layout(*d);
    char *ws = (char *)workspace;
    FitnessArgs a = {};
    a.P = d->P; a.J = d->J; a.N = d->N; a.Gm = d->Gm; a.Gs = d->Gs; a.flags = d->flags;
    a.m_grid = m_grid; a.job_params = job_params;
    a.status = (int32_t *)(ws + L.status);
    a.rs = (double *)(ws + L.rs);
    a.rsf = (float *)(ws + L.rsf);
    a.rk = (double *)(ws + L.rk);
    a.tg = (double2 *)(ws + L.tg);
    a.lntg = (double *)(ws + L.lntg);
    a.pu = (double *)(ws + L.pu);
    a.qh5 = (double *)(ws + L.qh5);
    a.ql5 = (double *)(ws + L.ql5);
    a.lt = (double *)(ws + L.lt);
    a.ca = (double2 *)(ws + L.ca);
    a.srange = (int32_t *)(ws + L.srange);
    a.k1 = (int32_t *)(ws + L.k1);
    a.gs_pad = ((d->Gs + 31) / 32) * 32;
    return a;
}

// tables_kernel and, for the grid sweeps (not the sampling argmax), last_kernel: everything the sweep of a (job, K, nodes) needs
static void launch_job_tables(const pollux_dims *d, const FitnessArgs &a, bool last_pass_tables, hipStream_t stream)
{
    long long table_items = (long long)d->J * d->Gm;
    if (table_items < a.gs_pad) table_items = a.gs_pad;
    if (table_items < kRecipTable) table_items = kRecipTable;
    hipLaunchKernelGGL(tables_kernel, dim3((unsigned)((table_items + 255) / 256)), dim3(256), 0, stream, a);
    const long long lt_rows = (long long)d->J * 2 * kTableK;
    if (last_pass_tables)
        hipLaunchKernelGGL(last_kernel, dim3((unsigned)((lt_rows / kLastRows + kWavesPerBlock - 1) / kWavesPerBlock)), dim3(256), 0, stream, a);
}

static int launch_queries(const pollux_dims *d, const double *job_params, const int32_t *m_grid, void *workspace,
                          const QueryArgs &q, hipStream_t stream)
{
    const FitnessArgs a = job_level_args(d, job_params, m_grid, workspace);
    launch_job_tables(d, a, true, stream);
    const long long queries = (long long)d->J * (q.mode == 0 ? q.max_nodes + 1 : 1);
    const dim3 grid((unsigned)((queries + kWavesPerBlock - 1) / kWavesPerBlock));
    const int ch = d->Gs <= 8 ? 8 : (d->Gs <= 16 ? 16 : 32);
    if (ch == 8) hipLaunchKernelGGL((queries_kernel<8>), grid, dim3(256), 0, stream, a, q);
    else if (ch == 16) hipLaunchKernelGGL((queries_kernel<16>), grid, dim3(256), 0, stream, a, q);
    else hipLaunchKernelGGL((queries_kernel<32>), grid, dim3(256), 0, stream, a, q);
    return hipGetLastError() == hipSuccess ? PX_OK : PX_E_HIP;
}

int launch_goodput_per_gpu(const pollux_dims *d, const double *job_params, const int32_t *m_grid, int gpus_per_node,
                           int max_nodes, void *workspace, double *per_gpu, hipStream_t stream)
{
    QueryArgs q = {};
    q.mode = 0; q.gpus_per_node = gpus_per_node; q.max_nodes = max_nodes; q.per_gpu = per_gpu;
    return launch_queries(d, job_params, m_grid, workspace, q, stream);
}

int launch_autoscale(int J, int max_nodes, const double *per_gpu, const int32_t *nodes_now, double U, double L,
                     int32_t *nodes_new, hipStream_t stream)
{
    hipLaunchKernelGGL(autoscale_kernel, dim3((unsigned)((J + 255) / 256)), dim3(256), 0, stream, J, max_nodes, per_gpu,
                       nodes_now, U, L, nodes_new);
    return hipGetLastError() == hipSuccess ? PX_OK : PX_E_HIP;
}

int launch_sim_tick(const pollux_dims *d, const double *job_params, const int32_t *m_grid, const int32_t *K,
                    const int32_t *nodes, const int32_t *changed, const double *target, double dt, double restart_delay,
                    void *workspace, double *progress, double *goodput, int32_t *finished, hipStream_t stream)
{
    QueryArgs q = {};
    q.mode = 1; q.K = K; q.nodes = nodes; q.changed = changed; q.target = target; q.dt = dt;
    q.restart_delay = restart_delay; q.progress = progress; q.goodput = goodput; q.finished = finished;
    return launch_queries(d, job_params, m_grid, workspace, q, stream);
}

__global__ void copy_status_kernel(const int32_t *__restrict__ from, int32_t *__restrict__ to)
{
    if (threadIdx.x == 0) *to = *from;
}

int launch_copy_status(const void *workspace, int32_t *status_out, hipStream_t stream)
{
    pollux_dims d = {1, 1, 1, 1, 1, 0, 0};
    const int32_t *word = (const int32_t *)((const char *)workspace + workspace_layout(d).status);
    hipLaunchKernelGGL(copy_status_kernel, dim3(1), dim3(64), 0, stream, word, status_out);
    return hipGetLastError() == hipSuccess ? PX_OK : PX_E_HIP;
}

int launch_fitness(const pollux_dims *d, const int32_t *population, const double *job_params, const int32_t *m_grid,
                   const int32_t *fair_share, const int32_t *current_alloc, const int32_t *node_capacity, double p,
                   double delta, void *workspace, double *fitness, int32_t *best_m, int32_t *best_s,
                   double *best_goodput, double *speedup, int32_t *violations, hipEvent_t sweep_start,
                   hipEvent_t sweep_stop, int first_rank, bool inherit_rows, hipStream_t stream)
{
    const WorkspaceLayout L = workspace_layout(*d);
    char *ws = (char *)workspace;
    FitnessArgs a = job_level_args(d, job_params, m_grid, workspace);
    a.population = population; a.fair_share = fair_share; a.current_alloc = current_alloc;
    a.node_capacity = node_capacity;
    a.p = p; a.delta = delta;
    a.clear_status = 1;
    a.denom = (double *)(ws + L.denom);
    a.factor = (double *)(ws + L.factor);
    a.running = (int32_t *)(ws + L.running);
    a.G = (double *)(ws + L.G);
    a.meta = (int32_t *)(ws + L.meta);
    a.memo = (MemoEntry *)(ws + L.memo);
    a.redo = (int32_t *)(ws + L.redo);
    a.curmask = (unsigned long long *)(ws + L.curmask);
    a.zeros = (int32_t *)(ws + L.zeros);
    a.colpack = (unsigned long long *)(ws + L.colpack);
    a.need_constraints = (violations != nullptr || !(d->flags & PX_FLAG_NO_CONSTRAINT_CHECK)) ? 1 : 0;
    // first_rank > 0: only the candidates of rank first_rank and beyond in the order the search step left in the
    // workspace, i.e. the slots it has just rewritten; the others keep the results they have
    const int P_eff = first_rank > 0 ? d->P - first_rank : d->P;
    if (first_rank > 0) {
        a.sel = (const int32_t *)(ws + L.order) + first_rank;
        a.n_sel = P_eff;
    }
    if (P_eff <= 0) return PX_OK;
    a.fitness = fitness; a.best_goodput = best_goodput; a.speedup = speedup;
    a.best_m = best_m; a.best_s = best_s; a.violations = violations;

    // unrolled s-chunk: the smallest of 8, 16, 32 that covers Gs (32 with several chunks beyond that)
    const int ch = d->Gs <= 8 ? 8 : (d->Gs <= 16 ? 16 : 32);
    const long long pairs = (long long)P_eff * d->J;
    // candidates per wavefront: enough wavefronts to fill the chip several times over
    long long per_wave = pairs / 25000;
    per_wave = per_wave < 1 ? 1 : (per_wave > kMaxCandPerWave ? kMaxCandPerWave : per_wave);
    a.cand_per_wave = (int)per_wave;
    a.cand_groups = (int)((P_eff + per_wave * kWavesPerBlock - 1) / (per_wave * kWavesPerBlock));
    const unsigned pair_blocks = (unsigned)(8 * ((d->J + 7) / 8) * a.cand_groups);

    const long long lt_rows = (long long)d->J * 2 * kTableK;
    const bool f32 = d->precision == 1;
    const bool memo = (d->flags & PX_FLAG_MEMOISE) != 0;
    const bool sampled = (d->flags & PX_FLAG_SAMPLE_M) != 0;       // fp64 only (checked by the caller)
    // The per-node counters start every call at zero.  A call that uses them leaves them at zero again
    // (candidates_kernel clears what it reads), so a call that keeps the job tables, whose caller guarantees an
    // untouched workspace and unchanged dimensions, does not clear them once more.
    const bool row1 = d->N <= 4 * kWave && (d->N & 3) == 0 && (((uintptr_t)population | (uintptr_t)current_alloc) & 15) == 0;
    const bool row4 = row1 && d->N <= kWave;        // four rows per load of a wavefront (cand_per_wave <= 16 holds)
    // memoised pass over rows of 65 to 256 entries: one workgroup per candidate, counters in LDS, fitness included
    const bool inherit = inherit_rows && first_rank > 0;
    // (not with row inheritance, whose rows to evaluate are listed per job, not per candidate)
    const bool candidate_pass = memo && !sampled && !f32 && row1 && !row4 && !inherit;
    if (inherit) {
        // the children of the step that has just run: unchanged rows take over their source's results; the others are
        // listed per job and go through the population pass below like any pair
        a.src_row = (const int32_t *)(ws + L.src_row);
        a.odd = (const int32_t *)(ws + L.odd);
        a.dirty_count = (int32_t *)(ws + L.dirty_count);
        a.dirty = (int32_t *)(ws + L.dirty);
        hipLaunchKernelGGL(inherit_kernel, dim3((unsigned)P_eff), dim3(256), 0, stream, a);
    }
    // done by tables_kernel, i.e. not by a call that keeps the job tables; the candidate pass keeps its counters on chip
    // and leaves those in memory alone, unless generations that inherit rows (and read them) are to follow
    a.clear_counters = (candidate_pass && !(d->flags & PX_FLAG_PAIR_RESULTS)) ? 0 : 1;
    if (!(d->flags & PX_FLAG_KEEP_JOB_TABLES)) {
        // everything that depends on the jobs only (not on the population)
        launch_job_tables(d, a, !sampled, stream);
        const dim3 job_grid((unsigned)((d->J + kWavesPerBlock - 1) / kWavesPerBlock));
        if (sampled) hipLaunchKernelGGL((jobs_kernel<0, false>), job_grid, dim3(256), 0, stream, a);
        else if (f32 && ch == 8) hipLaunchKernelGGL((jobs_kernel<8, true>), job_grid, dim3(256), 0, stream, a);
        else if (f32) hipLaunchKernelGGL((jobs_kernel<16, true>), job_grid, dim3(256), 0, stream, a);
        else if (ch == 8) hipLaunchKernelGGL((jobs_kernel<8, false>), job_grid, dim3(256), 0, stream, a);
        else if (ch == 16) hipLaunchKernelGGL((jobs_kernel<16, false>), job_grid, dim3(256), 0, stream, a);
        else hipLaunchKernelGGL((jobs_kernel<32, false>), job_grid, dim3(256), 0, stream, a);
        if (memo) {
            const dim3 memo_grid((unsigned)((lt_rows + kWavesPerBlock - 1) / kWavesPerBlock));
            if (sampled) hipLaunchKernelGGL((memo_kernel<0, false>), memo_grid, dim3(256), 0, stream, a);
            else if (f32 && ch == 8) hipLaunchKernelGGL((memo_kernel<8, true>), memo_grid, dim3(256), 0, stream, a);
            else if (f32) hipLaunchKernelGGL((memo_kernel<16, true>), memo_grid, dim3(256), 0, stream, a);
            else if (ch == 8) hipLaunchKernelGGL((memo_kernel<8, false>), memo_grid, dim3(256), 0, stream, a);
            else if (ch == 16) hipLaunchKernelGGL((memo_kernel<16, false>), memo_grid, dim3(256), 0, stream, a);
            else hipLaunchKernelGGL((memo_kernel<32, false>), memo_grid, dim3(256), 0, stream, a);
        }
    }
    if (sweep_start) (void)hipEventRecord(sweep_start, stream);
    const bool whole = d->Gm % kWave == 0;
    const bool near = a.gs_pad <= kNearRecips;      // the kernels keep reciprocals and thresholds of all counts in LDS
#define PX_LAUNCH_PAIRS(CH, F32, MEMO, ROW1, WHOLE, ROW4)                                                               \
    do {                                                                                                                \
        if (a.dirty) hipLaunchKernelGGL((pairs_kernel<CH, F32, MEMO, ROW1, WHOLE, ROW4, 2>), dim3(pair_blocks), dim3(256), 0, stream, a); \
        else if (a.sel) hipLaunchKernelGGL((pairs_kernel<CH, F32, MEMO, ROW1, WHOLE, ROW4, 1>), dim3(pair_blocks), dim3(256), 0, stream, a); \
        else hipLaunchKernelGGL((pairs_kernel<CH, F32, MEMO, ROW1, WHOLE, ROW4, 0>), dim3(pair_blocks), dim3(256), 0, stream, a); \
    } while (0)
    // the instance for the row length (four rows per load, one row per load, any) and the grid (whole groups of 64 batch sizes or not)
#define PX_LAUNCH_PAIRS_GRID(CH, F32)                                          \
    do {                                                                       \
        if (memo && row4) PX_LAUNCH_PAIRS(CH, F32, true, true, false, true);   \
        else if (memo && row1) PX_LAUNCH_PAIRS(CH, F32, true, true, false, false); \
        else if (memo) PX_LAUNCH_PAIRS(CH, F32, true, false, false, false);    \
        else if (row4 && whole && near) PX_LAUNCH_PAIRS(CH, F32, false, true, true, true); \
        else if (row1 && whole) PX_LAUNCH_PAIRS(CH, F32, false, true, true, false); \
        else if (row1) PX_LAUNCH_PAIRS(CH, F32, false, true, false, false);    \
        else PX_LAUNCH_PAIRS(CH, F32, false, false, false, false);             \
    } while (0)
    if (candidate_pass) {
        const dim3 memo_grid((unsigned)P_eff);
#define PX_LAUNCH_MEMO_CANDIDATES(CH)                                                                                 \
    do {                                                                                                              \
        if (d->flags & PX_FLAG_PAIR_RESULTS) {                                                                        \
            hipLaunchKernelGGL((memo_candidates_kernel<CH, false, true>), memo_grid, dim3(kCandThreads), 0, stream, a); \
            hipLaunchKernelGGL((memo_candidates_kernel<CH, true, true>), memo_grid, dim3(kCandThreads), 0, stream, a); \
        } else {                                                                                                      \
            hipLaunchKernelGGL((memo_candidates_kernel<CH, false, false>), memo_grid, dim3(kCandThreads), 0, stream, a); \
            hipLaunchKernelGGL((memo_candidates_kernel<CH, true, false>), memo_grid, dim3(kCandThreads), 0, stream, a); \
        }                                                                                                             \
    } while (0)
        if (ch == 8) PX_LAUNCH_MEMO_CANDIDATES(8);
        else if (ch == 16) PX_LAUNCH_MEMO_CANDIDATES(16);
        else PX_LAUNCH_MEMO_CANDIDATES(32);
#undef PX_LAUNCH_MEMO_CANDIDATES
        if (sweep_stop) (void)hipEventRecord(sweep_stop, stream);
        return hipGetLastError() == hipSuccess ? PX_OK : PX_E_HIP;
    } else if (sampled) {
        if (memo) PX_LAUNCH_PAIRS(0, false, true, false, false, false);
        else PX_LAUNCH_PAIRS(0, false, false, false, false, false);
    } else if (f32) {
        if (ch == 8) PX_LAUNCH_PAIRS_GRID(8, true);
        else PX_LAUNCH_PAIRS_GRID(16, true);
    } else if (ch == 8) {
        PX_LAUNCH_PAIRS_GRID(8, false);
    } else if (ch == 16) {
        PX_LAUNCH_PAIRS_GRID(16, false);
    } else {
        PX_LAUNCH_PAIRS_GRID(32, false);
    }
#undef PX_LAUNCH_PAIRS_GRID
#undef PX_LAUNCH_PAIRS
    if (sweep_stop) (void)hipEventRecord(sweep_stop, stream);
    if (f32) hipLaunchKernelGGL(candidates_kernel<float>, dim3((unsigned)P_eff), dim3(kCandThreads), 0, stream, a);
    else hipLaunchKernelGGL(candidates_kernel<double>, dim3((unsigned)P_eff), dim3(kCandThreads), 0, stream, a);
    return hipGetLastError() == hipSuccess ? PX_OK : PX_E_HIP;
}

}  // namespace px
