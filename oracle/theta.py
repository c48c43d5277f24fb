"""CPU checker for the online fitting of theta_sys (Pollux, arXiv 2008.12260, Sec. 4.1
"Online model fitting" and "Prior-driven exploration").

TEST INFRASTRUCTURE ONLY: imported by tests and by the CPU-baseline leg of the benchmark.

A job has recorded tuples (a, m, s, T_iter); of an allocation a the model sees K = SUM(a) and
the number of nodes occupied (Eq. 9).  theta_sys = (alpha_grad, beta_grad, alpha_sync^local,
beta_sync^local, alpha_sync^node, beta_sync^node, gamma) is fitted by minimising the root mean
squared logarithmic error between Eq. 11 and the recorded T_iter with L-BFGS-B (scipy's, the
routine the paper names), every alpha and beta >= 0 and 1 <= gamma <= 10.

Everything is plain fp64 numpy written from the equations: Eq. 8 (T_grad), Eq. 9 (T_sync),
Eq. 10 (overlap), Eq. 11 (accumulation).  The gradient is the analytic derivative of the same
expressions (tests compare it with finite differences).

Readings
  * Priors.  The text sets alpha_sync^local = 0 until the job has used more than one GPU, "alpha_sync^local =
    beta_sync^local = 0" until it has used more than one node, and beta_sync^local = beta_sync^node = 0 until it has
    used more than two GPUs.  The middle clause repeats the local pair where only the node pair makes sense (a
    job on one node has no evidence about the node pair, and plenty about the local one), so it is read as
    alpha_sync^node = beta_sync^node = 0.  With at most one GPU ever used nothing is known about either pair
    and all four are 0.  A parameter a prior fixes stays at 0 through the fit.
  * Start.  The paper gives no starting point, and the error has several local minima, so the checker has a
    start policy of its own (the GPU library has another; neither is the paper's).  Two base points:
    "tmin", from T_min = the smallest recorded T_iter / (s + 1): alpha_grad = T_min / 2, beta_grad =
    T_min / (2 m at that record), alpha_sync = T_min / 10, beta_sync = T_min / 100; and "linear", the
    non-negative least-squares solution of the model at gamma = 1, where Eq. 11 is linear in the six alphas and
    betas (relative residuals; scipy's nnls), with every free sync parameter raised to at least T_min / 100.
    STARTS lists (base, factor on the four sync parameters, gamma) combinations; fit(n_starts = n) runs L-BFGS-B
    from the first n and keeps the best end point.  Sync parameters must start above 0: at T_sync = 0 and gamma > 1
    the derivative of Eq. 10 with respect to T_sync vanishes and a descent method never leaves 0.
  * Local minima.  Which minimum a local method ends in depends on the method and the start.  The checks
    against the GPU library therefore pin the objective, the constraints and stationarity exactly and compare the
    attained minimum statistically ("parity partial" for the choice among local minima).
  * Scale.  The unknowns differ by four orders of magnitude (beta_grad ~ 1e-4 s/example, gamma ~ 2), so the
    minimiser works on theta / start (gamma unscaled); the minimum is the same.
"""
from __future__ import annotations

import numpy as np
from scipy.optimize import minimize

NTHETA = 7
ALPHA_G, BETA_G, ALPHA_SL, BETA_SL, ALPHA_SN, BETA_SN, GAMMA = range(7)
T_GRAD_FLOOR = 1e-12        # keeps ln T_grad finite if the minimiser ever tries alpha_grad = beta_grad = 0


def t_iter(theta, K, nodes, m, s):
    """Eq. 11 with Eq. 8-10 for arrays of records; returns (T_iter, T_grad, T_sync)."""
    theta = np.asarray(theta, np.float64)
    K, nodes, m, s = (np.asarray(x, np.float64) for x in (K, nodes, m, s))
    tg = np.maximum(theta[ALPHA_G] + theta[BETA_G] * m, T_GRAD_FLOOR)                      # Eq. 8
    ts = np.where(K <= 1, 0.0,                                                              # Eq. 9
                  np.where(nodes == 1, theta[ALPHA_SL] + theta[BETA_SL] * (K - 2),
                           theta[ALPHA_SN] + theta[BETA_SN] * (K - 2)))
    g = theta[GAMMA]
    with np.errstate(divide="ignore", invalid="ignore"):
        last = np.where(ts == 0.0, tg, np.power(np.power(tg, g) + np.power(ts, g), 1.0 / g))   # Eq. 10
    return s * tg + last, tg, ts                                                            # Eq. 11


def rmsle(theta, K, nodes, m, s, T):
    """Root mean squared logarithmic error between Eq. 11 and the recorded iteration times."""
    pred, _, _ = t_iter(theta, K, nodes, m, s)
    r = np.log(pred) - np.log(np.asarray(T, np.float64))
    return float(np.sqrt(np.mean(r * r)))


def residuals_and_jacobian(theta, K, nodes, m, s, T):
    """r_o = ln T_pred - ln T_obs and d r_o / d theta (analytic)."""
    theta = np.asarray(theta, np.float64)
    K, nodes, m, s, T = (np.asarray(x, np.float64) for x in (K, nodes, m, s, T))
    pred, tg, ts = t_iter(theta, K, nodes, m, s)
    g = theta[GAMMA]
    has_sync = ts > 0.0
    with np.errstate(divide="ignore", invalid="ignore"):
        last = pred - s * tg
        # d last / d T_grad = (T_grad / last)^(g-1), d last / d T_sync = (T_sync / last)^(g-1)
        dl_dtg = np.where(has_sync, np.power(tg / last, g - 1.0), 1.0)
        dl_dts = np.where(has_sync, np.power(ts / last, g - 1.0), 1.0 if g == 1.0 else 0.0)
        # d ln last / d g = (w_g ln T_grad + w_s ln T_sync) / g - ln(T_grad^g + T_sync^g) / g^2
        pg, ps = np.power(tg, g), np.power(ts, g)
        wsum = pg + ps
        dlnl_dg = np.where(has_sync,
                           (pg * np.log(tg) + ps * np.log(np.where(has_sync, ts, 1.0))) / (g * wsum) - np.log(wsum) / (g * g),
                           0.0)
    one_gpu = K <= 1
    local = (~one_gpu) & (nodes == 1)
    node = (~one_gpu) & (nodes != 1)
    J = np.zeros((T.size, NTHETA))
    J[:, ALPHA_G] = s + dl_dtg
    J[:, BETA_G] = (s + dl_dtg) * m
    J[:, ALPHA_SL] = np.where(local, dl_dts, 0.0)
    J[:, BETA_SL] = np.where(local, dl_dts * (K - 2), 0.0)
    J[:, ALPHA_SN] = np.where(node, dl_dts, 0.0)
    J[:, BETA_SN] = np.where(node, dl_dts * (K - 2), 0.0)
    J[:, GAMMA] = last * dlnl_dg
    J /= pred[:, None]
    return np.log(pred) - np.log(T), J


def rmsle_and_gradient(theta, K, nodes, m, s, T):
    r, J = residuals_and_jacobian(theta, K, nodes, m, s, T)
    f = float(np.sqrt(np.mean(r * r)))
    if f == 0.0:
        return 0.0, np.zeros(NTHETA)
    return f, (J.T @ r) / (r.size * f)


def prior_fixed(K, nodes):
    """Which parameters the exploration priors hold at 0 for a job with these records (see Readings)."""
    K, nodes = np.asarray(K), np.asarray(nodes)
    max_k = int(K.max()) if K.size else 0
    max_nodes = int(nodes.max()) if nodes.size else 0
    fixed = np.zeros(NTHETA, bool)
    if max_k <= 1:
        fixed[[ALPHA_SL, BETA_SL, ALPHA_SN, BETA_SN]] = True
    if max_nodes <= 1:
        fixed[[ALPHA_SN, BETA_SN]] = True
    if max_k <= 2:
        fixed[[BETA_SL, BETA_SN]] = True
    return fixed


def start_point(K, nodes, m, s, T):
    """The "tmin" base point (see Readings)."""
    m, s, T = (np.asarray(x, np.float64) for x in (m, s, T))
    per_pass = T / (s + 1.0)
    o = int(np.argmin(per_pass))                    # first record attaining the minimum
    t_min = per_pass[o]
    theta = np.array([t_min / 2, t_min / (2 * m[o]), t_min / 10, t_min / 100, t_min / 10, t_min / 100, 2.0])
    theta[prior_fixed(K, nodes)] = 0.0
    return theta


def linear_start(K, nodes, m, s, T):
    """The "linear" base point: at gamma = 1 Eq. 10 is T_grad + T_sync, so Eq. 11 is linear in the alphas and betas;
    their non-negative least-squares fit to the records (relative residuals), gamma = 2 as a placeholder."""
    from scipy.optimize import nnls
    K, nodes, m, s, T = (np.asarray(x, np.float64) for x in (K, nodes, m, s, T))
    one_gpu = K <= 1
    local = ((~one_gpu) & (nodes == 1)).astype(np.float64)
    node = ((~one_gpu) & (nodes != 1)).astype(np.float64)
    A = np.stack([s + 1.0, (s + 1.0) * m, local, local * (K - 2), node, node * (K - 2)], axis=1) / T[:, None]
    fixed = prior_fixed(K, nodes)
    free = np.flatnonzero(~fixed[:6])
    col = np.maximum(np.linalg.norm(A[:, free], axis=0), 1e-300)          # columns differ by orders of magnitude
    x, _ = nnls(A[:, free] / col, np.ones(T.size))
    theta = np.zeros(NTHETA)
    theta[free] = x / col
    t_min = float(np.min(T / (s + 1.0)))
    for i in (ALPHA_SL, BETA_SL, ALPHA_SN, BETA_SN):
        if not fixed[i]:
            theta[i] = max(theta[i], t_min / 100)
    if theta[ALPHA_G] + theta[BETA_G] <= 0.0:
        theta[ALPHA_G] = t_min / 2
    theta[GAMMA] = 2.0
    return theta


# (base point, factor on the four sync parameters, gamma) of the starts, in the order they are tried
STARTS = (("tmin", 1.0, 2.0), ("linear", 1.0, 2.0), ("linear", 1.0, 5.0), ("tmin", 4.0, 1.3), ("tmin", 0.25, 4.0),
          ("linear", 3.0, 1.3), ("tmin", 0.25, 1.3))


def fit(K, nodes, m, s, T, start=None, max_iter=2000, n_starts=1):
    """Sec. 4.1: minimise the RMSLE with L-BFGS-B under the box constraints and the priors.

    With `start` given, one run from there.  Otherwise the first n_starts entries of STARTS are tried and the best
    end point is kept, the earliest on ties.  Returns (theta, rmsle, scipy's result object)."""
    K, nodes, m, s, T = (np.asarray(x) for x in (K, nodes, m, s, T))
    if start is not None:
        x = np.asarray(start, np.float64).copy()
        return _fit_from(K, nodes, m, s, T, x, x.copy(), max_iter)
    bases = {"tmin": start_point(K, nodes, m, s, T)}
    best = None
    for base_name, factor, gamma0 in STARTS[:n_starts]:
        if base_name not in bases:
            bases[base_name] = linear_start(K, nodes, m, s, T)
        x = bases[base_name].copy()
        x[ALPHA_SL:BETA_SN + 1] *= factor
        x[GAMMA] = gamma0
        out = _fit_from(K, nodes, m, s, T, x, bases[base_name], max_iter)
        if best is None or out[1] < best[1]:
            best = out
    return best


def _fit_from(K, nodes, m, s, T, theta0, scale_from, max_iter):
    fixed = prior_fixed(K, nodes)
    theta0[fixed] = 0.0
    scale = np.where((scale_from > 0) & ~fixed, scale_from, 1.0)
    scale[GAMMA] = 1.0
    bounds = [(0.0, 0.0) if fixed[i] else (0.0, None) for i in range(6)] + [(1.0, 10.0)]

    def fun(z):
        f, g = rmsle_and_gradient(z * scale, K, nodes, m, s, T)
        return f, g * scale

    res = minimize(fun, theta0 / scale, jac=True, method="L-BFGS-B", bounds=bounds,
                   options=dict(maxiter=max_iter, maxfun=10 * max_iter, ftol=1e-15, gtol=1e-10, maxcor=20))
    theta = res.x * scale
    theta[fixed] = 0.0
    return theta, rmsle(theta, K, nodes, m, s, T), res
