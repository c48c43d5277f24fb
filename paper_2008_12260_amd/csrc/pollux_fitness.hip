// Fitness evaluation of a population of allocation matrices on gfx950.
//
// Pollux (arXiv 2008.12260): goodput model Sec. 3 (Eq. 4), statistical
// efficiency Sec. 3.1 (Eq. 6), throughput Sec. 3.2 (Eq. 7-11), per-job tuning
// Sec. 4.1 (Eq. 13), SPEEDUP / FITNESS_p, re-allocation penalty and
// interference avoidance Sec. 4.2 (Eq. 14-15).
//
// Kernels
//   tables_kernel     per job and grid point: T_grad(m) (Eq. 8) and ln T_grad;
//                     reciprocals 1/(s+1); clears the status word
//   jobs_kernel       per job (one wavefront): parameter checks, restart
//                     factor, fair-share goodput (denominator of Eq. 15)
//   pairs_kernel      per (candidate, job) (one wavefront): row reduce, sweep
//                     of the (m, s) grid, argmax, SPEEDUP
//   candidates_kernel per candidate (one workgroup): constraint check and the
//                     generalized mean
//
// How one wavefront sweeps the grid of a (candidate, job) pair.  Lane l owns
// the batch sizes m_i, i = l, l+64, ...; it walks s = 0..Gs-1.  Dividing Eq. 4
// through by M gives
//     GOODPUT = (phi + M0) / h,   h(m, s) = T_iter(m, s) * (1 + phi / M),
// and with u = phi/(K m), last = (T_grad^g + T_sync^g)^(1/g):
//     h(m, s) = (last + u T_grad) + s T_grad + (last - T_grad) u / (s + 1),
// two fused multiply-adds per grid point with every term non-negative.  The
// argmax of GOODPUT is the argmin of h over the feasible points.  The lane
// keeps the minimum with one v_min_f64 per point: the low five mantissa bits of
// h are replaced by s (so the minimum carries its own index and equal values
// resolve to the smaller s), and infeasible points get their exponent forced to
// the top of the range.  The perturbation is 2^-47 relative; the point each lane
// elects is then evaluated again with the formulas in the paper's own order
// (separate multiply and add, IEEE division), and the wave-wide argmax is taken
// over those values with ties going to the lowest flat index, so the reported
// goodput and the choice among lanes do not depend on the fast form.
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

namespace px {

struct FitnessArgs {
    int P, J, N, Gm, Gs, flags;
    const int32_t *population, *m_grid, *fair_share, *current_alloc, *node_capacity;
    const double *job_params;
    double p, delta;
    // workspace
    int32_t *status;
    double *rs, *tg, *lntg, *denom, *factor, *S;
    int32_t *running, *nodes;
    // outputs
    double *fitness, *best_goodput, *speedup;
    int32_t *best_m, *best_s, *violations;
};

struct Job {
    double alpha_g, beta_g, alpha_sl, beta_sl, alpha_sn, beta_sn, gamma, inv_gamma, phi, M0, Mmax, a;
};

__device__ __forceinline__ Job load_job(const double *__restrict__ jp, int J, int j)
{
    Job q;
    q.alpha_g = jp[(size_t)PX_ALPHA_G * J + j];
    q.beta_g = jp[(size_t)PX_BETA_G * J + j];
    q.alpha_sl = jp[(size_t)PX_ALPHA_SL * J + j];
    q.beta_sl = jp[(size_t)PX_BETA_SL * J + j];
    q.alpha_sn = jp[(size_t)PX_ALPHA_SN * J + j];
    q.beta_sn = jp[(size_t)PX_BETA_SN * J + j];
    q.gamma = jp[(size_t)PX_GAMMA * J + j];
    q.inv_gamma = 1.0 / q.gamma;
    q.phi = jp[(size_t)PX_PHI * J + j];
    q.M0 = jp[(size_t)PX_M0 * J + j];
    q.Mmax = jp[(size_t)PX_MMAX * J + j];
    q.a = q.phi + q.M0;
    return q;
}

// ---- tables ------------------------------------------------------------------

__global__ void __launch_bounds__(256) tables_kernel(FitnessArgs a)
{
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t == 0) *a.status = 0;
    if (t < a.Gs) a.rs[t] = 1.0 / (double)(t + 1);
    if (t < a.J * a.Gm) {
        int j = t / a.Gm;
        double m = (double)a.m_grid[t];
        double tg = a.job_params[(size_t)PX_ALPHA_G * a.J + j] + a.job_params[(size_t)PX_BETA_G * a.J + j] * m;   // Eq. 8
        a.tg[t] = tg;
        a.lntg[t] = log(tg);
    }
}

// ---- the sweep of one (job, K, nodes) ----------------------------------------

struct Best {
    double goodput;   // maximum of Eq. 4 over the grid, 0 if nothing is feasible
    int m, s;         // batch size and accumulation steps attaining it, -1/-1 if none
};

// Exact integer bounds on x = s + 1 from M0 <= Km * x <= Mmax, from a quotient that may be off by one.
__device__ __forceinline__ void feasible_range(double Km, double rKm, double M0, double Mmax, int &lo, int &hi)
{
    double qh = floor(Mmax * rKm);
    if (Km * (qh + 1.0) <= Mmax) qh += 1.0;
    if (Km * qh > Mmax) qh -= 1.0;
    double ql = ceil(M0 * rKm);
    if (Km * (ql - 1.0) >= M0) ql -= 1.0;
    if (Km * ql < M0) ql += 1.0;
    ql = fmin(fmax(ql, 1.0), 1073741824.0);
    qh = fmin(fmax(qh, 0.0), 1073741824.0);
    lo = (int)ql;
    hi = (int)qh;
}

// Eq. 4 at one grid point, in the paper's order of operations (no contraction).
__device__ __forceinline__ double goodput_point(const Job &q, double Km, double tg, double last, int s)
{
    double M = Km * (double)(s + 1);
    double t_iter = (double)s * tg + last;                       // Eq. 11
    double throughput = M / t_iter;                              // Eq. 7
    double efficiency = q.a / (q.phi + M);                       // Eq. 6
    return throughput * efficiency;                              // Eq. 4
}

// All 64 lanes call this with the same (job, K, nodes).  Every lane returns the same result.
__device__ __forceinline__ Best sweep(const Job &q, const int32_t *__restrict__ mg, const double *__restrict__ tgv,
                                      const double *__restrict__ lntgv, const double *__restrict__ rs, int Gm, int Gs,
                                      int K, int nodes)
{
    Best out = {0.0, -1, -1};
    if (K <= 0) return out;
    const int lane = lane_id();
    const double Kd = (double)K;
    // Eq. 9
    double ts = 0.0;
    if (K > 1) ts = (nodes == 1) ? q.alpha_sl + q.beta_sl * (double)(K - 2) : q.alpha_sn + q.beta_sn * (double)(K - 2);
    const int mode = (ts == 0.0) ? 0 : (q.gamma == 1.0 ? 1 : 2);
    const double lnts = (mode == 2) ? log(ts) : 0.0;

    double kbest = __builtin_inf();   // smallest key seen by this lane
    int ibest = -1, sbest = -1;
    double last_best = 0.0, tg_best = 0.0, Km_best = 0.0;
    int m_best = -1;

    for (int i0 = 0; i0 < Gm; i0 += kWave) {
        const int i = i0 + lane;
        const bool active = i < Gm;
        const int m = active ? mg[i] : 0;
        const double tg = active ? tgv[i] : 1.0;
        double last;                                             // last pass of Eq. 10
        if (mode == 0) {
            last = tg;
        } else if (mode == 1) {
            last = tg + ts;
        } else {
            double d = (active ? lntgv[i] : 0.0) - lnts;
            double e = exp(-q.gamma * fabs(d));
            last = fmax(tg, ts) * exp(log1p(e) * q.inv_gamma);
        }
        const bool usable = active && m > 0;
        const double Km = usable ? Kd * (double)m : 1.0;
        const double rKm = 1.0 / Km;
        int lo, hi;
        feasible_range(Km, rKm, q.M0, q.Mmax, lo, hi);
        if (!usable) { lo = 1; hi = 0; }
        const double u = q.phi * rKm;
        const double A0 = fma(u, tg, last);
        const double B0 = (last - tg) * u;

        for (int s0 = 0; s0 < Gs; s0 += 32) {
            // bit b of `bad` is set when s = s0 + b is infeasible for this lane
            int first = lo - 1 - s0, lastb = hi - 1 - s0;
            first = first < 0 ? 0 : first;
            lastb = lastb > 31 ? 31 : lastb;
            uint32_t ok = (first <= lastb) ? (uint32_t)((0xFFFFFFFFu >> (31 - lastb)) & (0xFFFFFFFFu << first)) : 0u;
            const int bad = (int)~ok;
            const int cnt = (Gs - s0) < 32 ? (Gs - s0) : 32;
            double kmin = __builtin_inf();
#pragma unroll 8
            for (int b = 0; b < cnt; ++b) {
                const int s = s0 + b;
                double h = fma(B0, rs[s], fma((double)s, tg, A0));
                int hh = __double2hiint(h), hl = __double2loint(h);
                hh |= __builtin_amdgcn_sbfe(bad, b, 1) & 0x7FE00000;      // infeasible: exponent to the top
                hl = (hl & ~31) | b;                                      // carry the index
                double key = __hiloint2double(hh, hl);
                kmin = key < kmin ? key : kmin;
            }
            if (kmin < kbest && kmin < 0x1p1022) {
                kbest = kmin;
                ibest = i;
                sbest = s0 + (__double2loint(kmin) & 31);
                last_best = last; tg_best = tg; Km_best = Km; m_best = m;
            }
        }
    }

    // the elected point of each lane, evaluated in the paper's order of operations
    double g = -1.0;
    int flat = 0x7FFFFFFF;
    if (ibest >= 0) {
        g = goodput_point(q, Km_best, tg_best, last_best, sbest);
        flat = ibest * Gs + sbest;
    }
    const double gmax = wave_max(g);
    if (!(gmax > 0.0)) return out;
    const int fmin_ = wave_min(g == gmax ? flat : 0x7FFFFFFF);
    const bool winner = (g == gmax) && (flat == fmin_);
    const uint64_t wmask = __ballot(winner);
    const int wl = __ffsll((unsigned long long)wmask) - 1;
    out.goodput = gmax;
    out.m = __shfl(m_best, wl);
    out.s = __shfl(sbest, wl);
    return out;
}

// ---- per job -----------------------------------------------------------------

__global__ void __launch_bounds__(256) jobs_kernel(FitnessArgs a)
{
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int j = blockIdx.x * (blockDim.x >> 6) + wave;
    if (j >= a.J) return;
    const int lane = lane_id();
    const Job q = load_job(a.job_params, a.J, j);
    const double w = a.job_params[(size_t)PX_WEIGHT * a.J + j];
    const double T = a.job_params[(size_t)PX_AGE_T * a.J + j];
    const double R = a.job_params[(size_t)PX_RESTARTS_R * a.J + j];
    int st = 0;
    if (!(q.gamma >= 1.0 && q.gamma <= 10.0) || !(q.alpha_g >= 0.0) || !(q.beta_g >= 0.0) || !(q.alpha_sl >= 0.0) ||
        !(q.beta_sl >= 0.0) || !(q.alpha_sn >= 0.0) || !(q.beta_sn >= 0.0) || !(q.phi > 0.0) || !(q.M0 >= 1.0) ||
        !(q.Mmax >= q.M0) || !(w >= 0.0) || !(q.Mmax <= 4503599627370496.0) || !(q.alpha_g + q.beta_g > 0.0))
        st |= PX_ST_BAD_PARAM;
    // re-allocation penalty factor of Sec. 4.2
    const double factor = (T - R * a.delta) / (T + a.delta);
    if (!(a.flags & PX_FLAG_NO_REALLOC_PENALTY) && !(T - R * a.delta > 0.0)) st |= PX_ST_BAD_RESTART;
    // does the job hold GPUs now?
    long long csum = 0;
    int neg = 0;
    for (int n = lane; n < a.N; n += kWave) {
        int c = a.current_alloc[(size_t)j * a.N + n];
        csum += c;
        neg |= c < 0;
    }
    const long long total = wave_sum(csum);
    if (__ballot(neg) != 0) st |= PX_ST_NEG_ALLOC;
    // denominator of Eq. 15: the same sweep at the fair-share allocation
    const Best fair = sweep(q, a.m_grid + (size_t)j * a.Gm, a.tg + (size_t)j * a.Gm, a.lntg + (size_t)j * a.Gm, a.rs,
                            a.Gm, a.Gs, a.fair_share[2 * j], a.fair_share[2 * j + 1]);
    if (!(fair.goodput > 0.0)) st |= PX_ST_ZERO_FAIR;
    if (lane == 0) {
        a.denom[j] = fair.goodput;
        a.factor[j] = factor;
        a.running[j] = total > 0;
        if (st) atomicOr(a.status, st);
    }
}

// ---- per (candidate, job) ------------------------------------------------------

__global__ void __launch_bounds__(256) pairs_kernel(FitnessArgs a)
{
    const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const long long pair = (long long)blockIdx.x * (blockDim.x >> 6) + wave;
    if (pair >= (long long)a.P * a.J) return;
    const int c = (int)(pair / a.J);
    const int j = (int)(pair - (long long)c * a.J);
    const int lane = lane_id();

    // row reduce: K = sum, nodes = #positive, changed = differs from the current row
    const int32_t *__restrict__ row = a.population + (size_t)pair * a.N;
    const int32_t *__restrict__ cur = a.current_alloc + (size_t)j * a.N;
    int ksum = 0, nodes = 0;
    bool changed = false, neg = false;
    for (int n0 = 0; n0 < a.N; n0 += kWave) {
        const int n = n0 + lane;
        const int v = n < a.N ? row[n] : 0;
        const int cv = n < a.N ? cur[n] : 0;
        ksum += v;
        nodes += __popcll(__ballot(v > 0));
        changed |= __ballot(v != cv) != 0;
        neg |= __ballot(v < 0) != 0;
    }
    const int K = wave_sum(ksum);

    const Job q = load_job(a.job_params, a.J, j);
    const Best best = sweep(q, a.m_grid + (size_t)j * a.Gm, a.tg + (size_t)j * a.Gm, a.lntg + (size_t)j * a.Gm, a.rs,
                            a.Gm, a.Gs, K, nodes);
    if (lane == 0) {
        // Eq. 15 and the re-allocation penalty
        const double d = a.denom[j];
        double s_j = d > 0.0 ? best.goodput / d : 0.0;
        if (!(a.flags & PX_FLAG_NO_REALLOC_PENALTY) && changed && a.running[j]) s_j = s_j * a.factor[j];
        a.S[pair] = s_j;
        a.nodes[pair] = nodes;
        a.best_m[pair] = best.m;
        a.best_s[pair] = best.s;
        if (a.best_goodput) a.best_goodput[pair] = best.goodput;
        if (a.speedup) a.speedup[pair] = s_j;
        if (neg) atomicOr(a.status, PX_ST_NEG_ALLOC);
    }
}

// ---- per candidate -------------------------------------------------------------

constexpr int kCandThreads = 256;

__device__ __forceinline__ double pmean_term(double s, double w, double p)
{
    if (p == 0.0) return w * log(s);      // log(0) = -inf
    return w * pow(s, p);                 // pow(0, p<0) = +inf
}

__global__ void __launch_bounds__(kCandThreads) candidates_kernel(FitnessArgs a)
{
    __shared__ double red_acc[kCandThreads];
    __shared__ double red_w[kCandThreads];
    __shared__ long long red_v[kCandThreads];
    const int c = blockIdx.x;
    const int t = threadIdx.x;
    const double *__restrict__ S = a.S + (size_t)c * a.J;
    const double *__restrict__ wt = a.job_params + (size_t)PX_WEIGHT * a.J;

    // generalized mean, Eq. 14: each thread sums its jobs in ascending order, then a fixed tree
    double acc = 0.0, wsum = 0.0;
    for (int j = t; j < a.J; j += kCandThreads) {
        acc += pmean_term(S[j], wt[j], a.p);
        wsum += wt[j];
    }
    red_acc[t] = acc;
    red_w[t] = wsum;

    // constraint check: thread <-> node, walk the jobs
    long long v = 0;
    const bool need_v = a.violations != nullptr || !(a.flags & PX_FLAG_NO_CONSTRAINT_CHECK);
    if (need_v) {
        const int32_t *__restrict__ A = a.population + (size_t)c * a.J * a.N;
        const int32_t *__restrict__ nodes = a.nodes + (size_t)c * a.J;
        for (int n = t; n < a.N; n += kCandThreads) {
            long long total = 0;
            int distributed = 0;
            for (int j = 0; j < a.J; ++j) {
                const int x = A[(size_t)j * a.N + n];
                total += x;
                distributed += (x > 0 && nodes[j] >= 2);
            }
            if (distributed > 1) v += distributed - 1;
            const long long over = total - (long long)a.node_capacity[n];
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
        const double mean = red_acc[0] / red_w[0];
        double f = (a.p == 0.0) ? exp(mean) : pow(mean, 1.0 / a.p);
        const long long V = red_v[0];
        if (a.violations) a.violations[c] = (int32_t)(V > 0x7FFFFFFF ? 0x7FFFFFFF : V);
        if (V > 0 && !(a.flags & PX_FLAG_NO_CONSTRAINT_CHECK)) f = -(double)V;
        a.fitness[c] = f;
    }
}

}  // namespace px

// ---- host side -----------------------------------------------------------------

namespace px {

int launch_fitness(const pollux_dims *d, const int32_t *population, const double *job_params, const int32_t *m_grid,
                   const int32_t *fair_share, const int32_t *current_alloc, const int32_t *node_capacity, double p,
                   double delta, void *workspace, double *fitness, int32_t *best_m, int32_t *best_s,
                   double *best_goodput, double *speedup, int32_t *violations, hipStream_t stream)
{
    const WorkspaceLayout L = workspace_layout(*d);
    char *ws = (char *)workspace;
    FitnessArgs a;
    a.P = d->P; a.J = d->J; a.N = d->N; a.Gm = d->Gm; a.Gs = d->Gs; a.flags = d->flags;
    a.population = population; a.m_grid = m_grid; a.fair_share = fair_share; a.current_alloc = current_alloc;
    a.node_capacity = node_capacity; a.job_params = job_params;
    a.p = p; a.delta = delta;
    a.status = (int32_t *)(ws + L.status);
    a.rs = (double *)(ws + L.rs);
    a.tg = (double *)(ws + L.tg);
    a.lntg = (double *)(ws + L.lntg);
    a.denom = (double *)(ws + L.denom);
    a.factor = (double *)(ws + L.factor);
    a.running = (int32_t *)(ws + L.running);
    a.S = (double *)(ws + L.S);
    a.nodes = (int32_t *)(ws + L.nodes);
    a.fitness = fitness; a.best_goodput = best_goodput; a.speedup = speedup;
    a.best_m = best_m; a.best_s = best_s; a.violations = violations;

    const long long table_items = (long long)d->J * d->Gm > d->Gs ? (long long)d->J * d->Gm : d->Gs;
    hipLaunchKernelGGL(tables_kernel, dim3((unsigned)((table_items + 255) / 256)), dim3(256), 0, stream, a);
    hipLaunchKernelGGL(jobs_kernel, dim3((unsigned)((d->J + 3) / 4)), dim3(256), 0, stream, a);
    const long long pairs = (long long)d->P * d->J;
    hipLaunchKernelGGL(pairs_kernel, dim3((unsigned)((pairs + 3) / 4)), dim3(256), 0, stream, a);
    hipLaunchKernelGGL(candidates_kernel, dim3((unsigned)d->P), dim3(kCandThreads), 0, stream, a);
    return hipGetLastError() == hipSuccess ? PX_OK : PX_E_HIP;
}

}  // namespace px
