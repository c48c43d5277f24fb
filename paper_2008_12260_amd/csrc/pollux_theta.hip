// Batched fitting of theta_sys on gfx950 (Pollux, arXiv 2008.12260, Sec. 4.1 "Online
// model fitting" and "Prior-driven exploration"): for every job, the seven throughput
// parameters (Eq. 12) that minimise the root mean squared logarithmic error between
// Eq. 11 and the job's recorded (K, nodes, m, s, T_iter) tuples, with every alpha and
// beta >= 0 and 1 <= gamma <= 10, and with the parameters the exploration priors hold
// at zero.
//
// One workgroup per job, one wavefront per starting point.  The lanes of a wavefront share the
// job's records; everything about the seven unknowns is the same in every lane.  The error is a sum of squares of
//     r_o = ln T_iter(theta; K_o, nodes_o, m_o, s_o) - ln T_o,
// so the minimiser is a damped Gauss-Newton (Levenberg-Marquardt) iteration on the box:
// per iteration the lanes form r_o and its seven partial derivatives, the wave reduces
// SUM r^2, J^T r (7 sums) and J^T J (28 sums) in a fixed butterfly order, every lane
// solves the damped 7 x 7 system on the variables that are free (not held by a prior,
// not at a bound with the gradient pointing outwards) by Cholesky factorisation, clips
// the step to the box and accepts it if SUM r^2 went down.  The unknowns are scaled by
// the starting point (they differ by four orders of magnitude).
//
// Eq. 10 is evaluated with the larger term factored out, as in the fitness kernels:
// with D = ln T_sync - ln T_grad and e = exp(-gamma |D|),
//     ln last = max(ln T_grad, ln T_sync) + log1p(e) / gamma,
//     w_s = T_sync^gamma / (T_grad^gamma + T_sync^gamma) = 1/(1+e) or e/(1+e),
//     d last / d T_grad = w_g last / T_grad,   d last / d T_sync = w_s last / T_sync,
//     d ln last / d gamma = (w_g ln T_grad + w_s ln T_sync) / gamma - ln(T_grad^gamma + T_sync^gamma) / gamma^2.

#include <hip/hip_runtime.h>
#include <math.h>
#include <stdint.h>

#include "../../include/pollux.h"
#include "pollux_device.h"
#include "pollux_host.h"
#include "pollux_math.h"

namespace px {

constexpr int kTheta = 7;                 // unknowns, in the order of the first seven PX_* rows
constexpr int kPacked = 28;               // lower triangle of a symmetric 7 x 7 matrix, row-major: (i, k <= i) at i(i+1)/2 + k
constexpr double kTgradFloor = 1e-12;     // keeps ln T_grad finite should alpha_grad = beta_grad = 0 ever be tried

struct FitArgs {
    int J, max_obs, max_iter, n_starts;
    const int32_t *count, *K, *nodes, *m, *s;
    const double *T, *init;
    double *theta, *rmsle;
    int32_t *iterations;
};

template <int STEP = 0>
__device__ __forceinline__ double wave_sum_f64(double v)
{
    v += exchange<STEP>(v);
    if constexpr (STEP < 5) return wave_sum_f64<STEP + 1>(v);
    return v;
}

__device__ __forceinline__ double uniform_f64(double v)
{
    return __hiloint2double(__builtin_amdgcn_readfirstlane(__double2hiint(v)),
                            __builtin_amdgcn_readfirstlane(__double2loint(v)));
}

// One recorded tuple in the form the iteration uses it.
struct Record {
    int K, nodes;
    double md, sd, lnT;
};

__device__ __forceinline__ Record load_record(const FitArgs &f, size_t at)
{
    Record r;
    r.K = f.K[at]; r.nodes = f.nodes[at];
    r.md = (double)f.m[at]; r.sd = (double)f.s[at];
    r.lnT = px_log(f.T[at]);
    return r;
}

// SUM r^2, J^T r and J^T J of one job at theta = z * scale.
struct Normal {
    double sse;
    double g[kTheta];
    double a[kPacked];
};

// mine: the record of lane l when the job has at most 64 of them (held: read once per job, kept in registers
// over all iterations); otherwise the records are read from memory in every evaluation.
__device__ __forceinline__ Normal normal_equations(const FitArgs &f, int j, int n, const double (&z)[kTheta],
                                                   const double (&scale)[kTheta], const Record &mine, bool held_records)
{
    const int lane = lane_id();
    double th[kTheta];
#pragma unroll
    for (int i = 0; i < kTheta; ++i) th[i] = z[i] * scale[i];
    const double gamma = th[PX_GAMMA], inv_gamma = 1.0 / gamma;

    Normal acc;
    acc.sse = 0.0;
#pragma unroll
    for (int i = 0; i < kTheta; ++i) acc.g[i] = 0.0;
#pragma unroll
    for (int i = 0; i < kPacked; ++i) acc.a[i] = 0.0;

    const size_t base = (size_t)j * f.max_obs;
    for (int o = lane; o < n; o += kWave) {
        const Record rec = held_records ? mine : load_record(f, base + o);
        const int K = rec.K, nodes = rec.nodes;
        const double md = rec.md, sd = rec.sd;
        const double lnT = rec.lnT;
        double tg = th[PX_ALPHA_G] + th[PX_BETA_G] * md;                                  // Eq. 8
        tg = tg > kTgradFloor ? tg : kTgradFloor;
        const bool local = K > 1 && nodes == 1, node = K > 1 && nodes != 1;
        const double km2 = (double)(K - 2);
        double ts = 0.0;                                                                  // Eq. 9
        if (local) ts = th[PX_ALPHA_SL] + th[PX_BETA_SL] * km2;
        if (node) ts = th[PX_ALPHA_SN] + th[PX_BETA_SN] * km2;
        double last = tg, dl_dtg = 1.0, dl_dts = gamma == 1.0 ? 1.0 : 0.0, dlnl_dg = 0.0;
        if (ts > 0.0) {                                                                   // Eq. 10
            const double lntg = px_log(tg), lnts = px_log(ts);
            const double d = lnts - lntg;
            const double e = px_exp(-gamma * fabs(d));
            const double l1p = px_log1p_unit(e);
            const double big = d >= 0.0 ? ts : tg, lnbig = d >= 0.0 ? lnts : lntg;
            last = big * px_exp(l1p * inv_gamma);
            const double w_small = px_div(e, 1.0 + e), w_big = px_div(1.0, 1.0 + e);
            const double w_s = d >= 0.0 ? w_big : w_small, w_g = d >= 0.0 ? w_small : w_big;
            dl_dtg = w_g * px_div(last, tg);
            dl_dts = w_s * px_div(last, ts);
            const double lnsum = gamma * lnbig + l1p;                                     // ln(T_grad^g + T_sync^g)
            dlnl_dg = (w_g * lntg + w_s * lnts) * inv_gamma - lnsum * inv_gamma * inv_gamma;
        }
        const double pred = sd * tg + last;                                               // Eq. 11
        const double r = px_log(pred) - lnT;
        const double inv_pred = px_div(1.0, pred);
        double d[kTheta];
        d[PX_ALPHA_G] = (sd + dl_dtg) * inv_pred;
        d[PX_BETA_G] = d[PX_ALPHA_G] * md;
        const double dts = dl_dts * inv_pred;
        d[PX_ALPHA_SL] = local ? dts : 0.0;
        d[PX_BETA_SL] = local ? dts * km2 : 0.0;
        d[PX_ALPHA_SN] = node ? dts : 0.0;
        d[PX_BETA_SN] = node ? dts * km2 : 0.0;
        d[PX_GAMMA] = last * dlnl_dg * inv_pred;
#pragma unroll
        for (int i = 0; i < kTheta; ++i) d[i] *= scale[i];
        acc.sse = px_fma(r, r, acc.sse);
#pragma unroll
        for (int i = 0; i < kTheta; ++i) {
            acc.g[i] = px_fma(d[i], r, acc.g[i]);
#pragma unroll
            for (int k = 0; k <= i; ++k) acc.a[i * (i + 1) / 2 + k] = px_fma(d[i], d[k], acc.a[i * (i + 1) / 2 + k]);
        }
    }
    Normal out;
    out.sse = uniform_f64(wave_sum_f64(acc.sse));
#pragma unroll
    for (int i = 0; i < kTheta; ++i) out.g[i] = uniform_f64(wave_sum_f64(acc.g[i]));
#pragma unroll
    for (int i = 0; i < kPacked; ++i) out.a[i] = uniform_f64(wave_sum_f64(acc.a[i]));
    return out;
}

// Solves (A + lambda diag(A)) x = -g on the free variables (bit i of `held` set: x_i = 0) by Cholesky
// factorisation of the packed lower triangle.  Returns false if a pivot is not positive.
__device__ __forceinline__ bool damped_step(const Normal &q, double lambda, unsigned held, double (&x)[kTheta])
{
    double l[kPacked];
    double b[kTheta];
#pragma unroll
    for (int i = 0; i < kTheta; ++i) {
        const bool hi = (held >> i) & 1u;
#pragma unroll
        for (int k = 0; k < i; ++k) l[i * (i + 1) / 2 + k] = (hi || ((held >> k) & 1u)) ? 0.0 : q.a[i * (i + 1) / 2 + k];
        const double dii = q.a[i * (i + 1) / 2 + i];
        l[i * (i + 1) / 2 + i] = hi ? 1.0 : dii + lambda * (dii > 1e-300 ? dii : 1e-300);
        b[i] = hi ? 0.0 : -q.g[i];
    }
    // (one division per pivot: the entries below it and both substitutions multiply by its reciprocal)
    double inv[kTheta];
    bool ok = true;
#pragma unroll
    for (int i = 0; i < kTheta; ++i) {
#pragma unroll
        for (int k = 0; k <= i; ++k) {
            double s = l[i * (i + 1) / 2 + k];
#pragma unroll
            for (int t = 0; t < k; ++t) s = px_fma(-l[i * (i + 1) / 2 + t], l[k * (k + 1) / 2 + t], s);
            if (k == i) {
                if (!(s > 0.0)) { ok = false; s = 1.0; }
                l[i * (i + 1) / 2 + i] = sqrt(s);
                inv[i] = 1.0 / l[i * (i + 1) / 2 + i];
            } else {
                l[i * (i + 1) / 2 + k] = s * inv[k];
            }
        }
    }
    // forward then backward substitution
#pragma unroll
    for (int i = 0; i < kTheta; ++i) {
        double s = b[i];
#pragma unroll
        for (int t = 0; t < i; ++t) s = px_fma(-l[i * (i + 1) / 2 + t], b[t], s);
        b[i] = s * inv[i];
    }
#pragma unroll
    for (int i = kTheta - 1; i >= 0; --i) {
        double s = b[i];
#pragma unroll
        for (int t = i + 1; t < kTheta; ++t) s = px_fma(-l[t * (t + 1) / 2 + i], x[t], s);
        x[i] = s * inv[i];
    }
    return ok;
}

constexpr int kMaxStarts = 5;

__global__ void __launch_bounds__(64 * kMaxStarts) fit_theta_kernel(FitArgs f)
{
    __shared__ double end_sse[kMaxStarts];
    __shared__ double end_z[kMaxStarts][kTheta];
    __shared__ int end_it[kMaxStarts];
    const int j = blockIdx.x;
    const int lane = lane_id();
    const int k = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));      // this wavefront's starting point
    const int n = f.count[j] < f.max_obs ? f.count[j] : f.max_obs;
    if (n <= 0) {
        if (k == 0 && lane < kTheta) f.theta[(size_t)lane * f.J + j] = lane == PX_GAMMA ? 1.0 : 0.0;
        if (k == 0 && lane == 0) {
            f.rmsle[j] = 0.0;
            if (f.iterations) f.iterations[j] = 0;
        }
        return;
    }
    const size_t base = (size_t)j * f.max_obs;

    // what the job has explored, and the record with the shortest time per pass (first one on ties)
    int max_k = 0, max_nodes = 0;
    double best = __builtin_inf();
    int best_o = 0x7FFFFFFF;
    for (int o = lane; o < n; o += kWave) {
        const int K = f.K[base + o], nd = f.nodes[base + o];
        max_k = K > max_k ? K : max_k;
        max_nodes = nd > max_nodes ? nd : max_nodes;
        const double per_pass = f.T[base + o] / (double)(f.s[base + o] + 1);
        if (per_pass < best) { best = per_pass; best_o = o; }
    }
    max_k = (int)wave_max((unsigned)max_k);
    max_nodes = (int)wave_max((unsigned)max_nodes);
    {
        // positive doubles order like their bit patterns
        const unsigned hi = (unsigned)__double2hiint(best), lo = (unsigned)__double2loint(best);
        const unsigned hmin = wave_min(hi);
        const unsigned lmin = wave_min(hi == hmin ? lo : 0xFFFFFFFFu);
        best_o = wave_min((hi == hmin && lo == lmin) ? best_o : 0x7FFFFFFF);
        best = __hiloint2double((int)hmin, (int)lmin);
    }
    const double t_min = uniform_f64(best);
    // the usual case, at most one record per lane: each lane keeps its record for the whole fit
    const bool held_records = n <= kWave;
    Record mine = {1, 1, 1.0, 0.0, 0.0};
    if (held_records && lane < n) mine = load_record(f, base + lane);
    const double m_at = (double)f.m[base + (size_t)__builtin_amdgcn_readfirstlane(best_o)];

    // priors (Sec. 4.1, "Prior-driven exploration"): parameters without evidence are held at zero
    unsigned prior = 0u;
    if (max_k <= 1) prior |= (1u << PX_ALPHA_SL) | (1u << PX_BETA_SL) | (1u << PX_ALPHA_SN) | (1u << PX_BETA_SN);
    if (max_nodes <= 1) prior |= (1u << PX_ALPHA_SN) | (1u << PX_BETA_SN);
    if (max_k <= 2) prior |= (1u << PX_BETA_SL) | (1u << PX_BETA_SN);
    // Held in a vector register on purpose: everything derived from it (the active set, the iterate) then lives in
    // vector registers, which this kernel has to spare, instead of in scalar registers, which it would spill.
    asm("" : "+v"(prior));

    double start[kTheta] = {t_min * 0.5, t_min / (2.0 * m_at), t_min / 10.0, t_min / 100.0, t_min / 10.0, t_min / 100.0, 2.0};
    if (f.init) {
#pragma unroll
        for (int i = 0; i < kTheta; ++i) start[i] = f.init[(size_t)i * f.J + j];
    }
    double scale[kTheta], lo[kTheta], hi[kTheta];
#pragma unroll
    for (int i = 0; i < kTheta; ++i) {
        if ((prior >> i) & 1u) start[i] = 0.0;
        scale[i] = (i != PX_GAMMA && start[i] > 0.0) ? start[i] : 1.0;
        lo[i] = i == PX_GAMMA ? 1.0 : 0.0;
        hi[i] = i == PX_GAMMA ? 10.0 : __builtin_inf();
    }

    // The error has several local minima (and a flat spot at T_sync = 0 when gamma > 1), so the iteration is
    // run from a few starting points, one per wavefront, and the best end point is kept (the first one on
    // ties).  Start 0 is the start itself.  Starts 1 and 2 first minimise with gamma held at 1, where
    // Eq. 11 is linear in the alphas and betas, then release gamma from 2 and from 5 with the sync
    // parameters raised to at least a tenth of their starting values.  Starts 3 and 4 scale the sync
    // parameters by 3 and 0.3 and begin at gamma = 1.2 and 5.
    {
        const bool two_phase = k == 1 || k == 2;
        const double sync_factor = (k == 3) ? 3.0 : (k == 4 ? 0.3 : 1.0);
        const double gamma0 = (k == 0) ? start[PX_GAMMA] : (k == 1 ? 2.0 : (k == 3 ? 1.2 : 5.0));
        // the default starting values of the sync parameters, in the units of z (used where one has to leave zero)
        const double sync_a = (t_min / 10.0), sync_b = (t_min / 100.0);
        double z[kTheta];
#pragma unroll
        for (int i = 0; i < kTheta; ++i) {
            double v = start[i];
            if (i >= PX_ALPHA_SL && i <= PX_BETA_SN) v *= sync_factor;
            if (i == PX_GAMMA) v = two_phase ? 1.0 : gamma0;
            v /= scale[i];
            z[i] = v < lo[i] ? lo[i] : (v > hi[i] ? hi[i] : v);
        }

        Normal cur;
        int it = 0;
        // The damped Gauss-Newton iteration from z, until it converges or the budget of steps is spent;
        // the variables in `hold` stay where they are.  Leaves the end point in z and its sums in cur.
        auto descend = [&](unsigned hold) {
            cur = normal_equations(f, j, n, z, scale, mine, held_records);
            double lambda = 1e-3;
            while (it < f.max_iter && cur.sse > 0.0) {
                ++it;
                unsigned held = hold;
#pragma unroll
                for (int i = 0; i < kTheta; ++i) {
                    if ((z[i] <= lo[i] && cur.g[i] > 0.0) || (z[i] >= hi[i] && cur.g[i] < 0.0)) held |= 1u << i;
                }
                // a free variable that sits on a bound and would be pushed across it joins the held set
                double step[kTheta];
                bool solved = false;
                for (int pass = 0; pass < kTheta + 1; ++pass) {
                    solved = damped_step(cur, lambda, held, step);
                    if (!solved) break;
                    unsigned more = 0u;
#pragma unroll
                    for (int i = 0; i < kTheta; ++i) {
                        if (!((held >> i) & 1u) && ((z[i] <= lo[i] && step[i] < 0.0) || (z[i] >= hi[i] && step[i] > 0.0))) more |= 1u << i;
                    }
                    if (!more) break;
                    held |= more;
                }
                if (!solved) {
                    lambda *= 10.0;
                    if (lambda > 1e15) break;
                    continue;
                }
                double zn[kTheta];
                double moved = 0.0;
#pragma unroll
                for (int i = 0; i < kTheta; ++i) {
                    double v = ((held >> i) & 1u) ? z[i] : z[i] + step[i];
                    v = v < lo[i] ? lo[i] : (v > hi[i] ? hi[i] : v);
                    zn[i] = v;
                    const double rel = fabs(v - z[i]) / (fabs(z[i]) + 1e-12);
                    moved = rel > moved ? rel : moved;
                }
                if (moved == 0.0) break;
                const Normal trial = normal_equations(f, j, n, zn, scale, mine, held_records);
                if (trial.sse < cur.sse) {
                    const double gain = (cur.sse - trial.sse) / cur.sse;
#pragma unroll
                    for (int i = 0; i < kTheta; ++i) z[i] = zn[i];
                    cur = trial;
                    lambda = lambda * 0.2 > 1e-15 ? lambda * 0.2 : 1e-15;
                    if (gain < 1e-13 && moved < 1e-9) break;
                } else {
                    lambda *= 5.0;
                    if (lambda > 1e15 || moved < 1e-15) break;
                }
            }
        };

        if (two_phase) {
            descend(prior | (1u << PX_GAMMA));
            z[PX_GAMMA] = gamma0;
#pragma unroll
            for (int i = PX_ALPHA_SL; i <= PX_BETA_SN; ++i) {
                const double least = 0.1 * ((i == PX_ALPHA_SL || i == PX_ALPHA_SN) ? sync_a : sync_b) / scale[i];
                if (!((prior >> i) & 1u) && z[i] < least) z[i] = least;
            }
        }
        descend(prior);
        // A sync pair that has ended at zero may only be stuck there: with T_sync = 0 and gamma > 1 the error
        // does not feel the pair at all (the flat spot).  It is put back to its default starting value once, the
        // others staying where they are, and the iteration is continued; the better end point is kept.
#pragma unroll
        for (int pair = 0; pair < 2; ++pair) {
            const int ia = pair == 0 ? PX_ALPHA_SL : PX_ALPHA_SN, ib = ia + 1;
            const bool stuck = !((prior >> ia) & 1u) && z[ia] == 0.0 && (((prior >> ib) & 1u) || z[ib] == 0.0);
            if (stuck && it < f.max_iter && cur.sse > 0.0) {
                double z_before[kTheta];
#pragma unroll
                for (int i = 0; i < kTheta; ++i) z_before[i] = z[i];
                const double sse_before = cur.sse;
                z[ia] = sync_a / scale[ia];
                descend(prior);
                if (!(cur.sse < sse_before)) {
#pragma unroll
                    for (int i = 0; i < kTheta; ++i) z[i] = z_before[i];
                    cur.sse = sse_before;
                }
            }
        }
        if (lane == 0) {
            end_sse[k] = cur.sse;
            end_it[k] = it;
#pragma unroll
            for (int i = 0; i < kTheta; ++i) end_z[k][i] = z[i];
        }
    }
    __syncthreads();
    if (k != 0) return;

    int best_k = 0, total_it = 0;
    for (int c = 0; c < f.n_starts; ++c) {
        total_it += end_it[c];
        if (end_sse[c] < end_sse[best_k]) best_k = c;
    }
    const double best_sse = end_sse[best_k];
    if (lane < kTheta) {
        double sc = 1.0;
#pragma unroll
        for (int i = 0; i < kTheta; ++i) {
            if (lane == i) sc = scale[i];
        }
        f.theta[(size_t)lane * f.J + j] = end_z[best_k][lane] * sc;
    }
    if (lane == 0) {
        f.rmsle[j] = sqrt(best_sse / (double)n);
        if (f.iterations) f.iterations[j] = total_it;
    }
}

int launch_fit_theta(int J, int max_obs, int max_iter, int n_starts, const int32_t *count, const int32_t *K, const int32_t *nodes,
                     const int32_t *m, const int32_t *s, const double *T, const double *init, double *theta,
                     double *rmsle, int32_t *iterations, hipStream_t stream)
{
    FitArgs f;
    f.J = J; f.max_obs = max_obs; f.max_iter = max_iter; f.n_starts = n_starts;
    f.count = count; f.K = K; f.nodes = nodes; f.m = m; f.s = s; f.T = T; f.init = init;
    f.theta = theta; f.rmsle = rmsle; f.iterations = iterations;
    hipLaunchKernelGGL(fit_theta_kernel, dim3((unsigned)J), dim3(64 * (unsigned)n_starts), 0, stream, f);
    return hipGetLastError() == hipSuccess ? PX_OK : PX_E_HIP;
}

}  // namespace px
