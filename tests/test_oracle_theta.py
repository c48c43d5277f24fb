"""Pins of the CPU checker for the fitting of theta_sys (Sec. 4.1): the objective against values worked out by
hand and against the goodput checker's own Eq. 11, the gradient against finite differences, the priors, and the
fit against records generated from known parameters."""
import numpy as np

import oracle as O
import oracle.theta as TH
import workloads as W

THETA = np.array([0.1, 0.001, 0.05, 0.01, 0.2, 0.02, 2.0])


def records(theta, n, max_k, rng, cap=4, sigma=0.0):
    K = rng.integers(1, max_k + 1, n)
    nodes = np.maximum(np.where(rng.uniform(size=n) < 0.7, -(-K // cap), np.minimum(K, rng.integers(1, 5, n))), 1)
    m = rng.choice([8, 16, 32, 64, 128, 256], n)
    s = rng.integers(0, 4, n)
    T, _, _ = TH.t_iter(theta, K, nodes, m, s)
    return K, nodes, m, s, T * np.exp(sigma * rng.standard_normal(n))


def test_iteration_time_matches_the_hand_derived_vectors():
    """T_iter of the vectors in tests/golden/goodput_vectors.txt (derived there from Eq. 8-11)."""
    for (K, nodes, m, s, gamma), want in [((1, 1, 100, 0, 2.0), 0.2), ((2, 1, 100, 0, 1.0), 0.25),
                                          ((2, 1, 100, 1, 2.0), 0.406155281281), ((4, 2, 50, 3, 3.0), 0.708127573469)]:
        th = THETA.copy()
        th[TH.GAMMA] = gamma
        got = TH.t_iter(th, [K], [nodes], [m], [s])[0][0]
        assert abs(got - want) <= 1e-11 * want


def test_iteration_time_is_the_one_the_goodput_checker_uses():
    rng = np.random.default_rng(1)
    jb = O.job(*THETA[:6], 2.7, 1000.0, 64.0, 4096.0)
    th = THETA.copy()
    th[TH.GAMMA] = 2.7
    for _ in range(200):
        K, nodes = int(rng.integers(1, 17)), int(rng.integers(1, 5))
        m, s = int(rng.integers(1, 300)), int(rng.integers(0, 6))
        want = O.titer(O.tgrad(jb.alpha_g, jb.beta_g, float(m)), O.tsync(jb, K, nodes), jb.gamma, s)
        assert abs(TH.t_iter(th, [K], [nodes], [m], [s])[0][0] - want) <= 1e-14 * want


def test_rmsle_closed_forms():
    rng = np.random.default_rng(2)
    K, nodes, m, s, T = records(THETA, 25, 16, rng)
    assert TH.rmsle(THETA, K, nodes, m, s, T) < 1e-15                       # the generating parameters fit exactly
    for c in (0.5, 1.25, 3.0):                                              # all times off by a factor c: |ln c|
        assert abs(TH.rmsle(THETA, K, nodes, m, s, T * c) - abs(np.log(c))) < 1e-13
    half = np.where(np.arange(25) % 2 == 0, 2.0, 1.0)                       # every other record off by 2
    want = np.sqrt(np.mean(np.log(half) ** 2))
    assert abs(TH.rmsle(THETA, K, nodes, m, s, T * half) - want) < 1e-13


def test_gradient_matches_central_differences():
    rng = np.random.default_rng(3)
    for trial in range(20):
        K, nodes, m, s, T = records(THETA, 30, 16, rng, sigma=0.05)
        x = THETA * np.exp(0.3 * rng.standard_normal(7))
        x[TH.GAMMA] = rng.uniform(1.0, 10.0) if trial else 1.0              # gamma = 1 once: the plain-sum branch
        f, g = TH.rmsle_and_gradient(x, K, nodes, m, s, T)
        for i in range(7):
            h = 1e-6 * max(abs(x[i]), 1e-3)
            xp, xm = x.copy(), x.copy()
            xp[i] += h
            xm[i] -= h
            if i == TH.GAMMA and x[i] == 1.0:
                continue                                                     # one-sided at the bound
            num = (TH.rmsle(xp, K, nodes, m, s, T) - TH.rmsle(xm, K, nodes, m, s, T)) / (2 * h)
            assert abs(g[i] - num) <= 1e-6 * max(abs(num), 1e-3 * np.max(np.abs(g))), (trial, i, g[i], num)


def test_priors_hold_unexplored_parameters_at_zero():
    rng = np.random.default_rng(4)
    names = {1: [2, 3, 4, 5], 2: [3, 5]}
    for max_k, zero in names.items():
        K, nodes, m, s, T = records(THETA, 30, max_k, rng, sigma=0.02)
        theta, f, _ = TH.fit(K, nodes, m, s, T)
        assert all(theta[i] == 0.0 for i in zero)
    K, nodes, m, s, T = records(THETA, 30, 4, rng, cap=4, sigma=0.02)
    nodes[:] = 1                                                            # up to four GPUs, one node only
    T = TH.t_iter(THETA, K, nodes, m, s)[0]
    theta, f, _ = TH.fit(K, nodes, m, s, T)
    assert theta[TH.ALPHA_SN] == 0.0 and theta[TH.BETA_SN] == 0.0 and theta[TH.ALPHA_SL] > 0.0
    assert np.array_equal(TH.prior_fixed([1, 1], [1, 1]), [False, False, True, True, True, True, False])
    assert np.array_equal(TH.prior_fixed([2, 1], [2, 1]), [False, False, False, True, False, True, False])
    assert np.array_equal(TH.prior_fixed([3, 1], [1, 1]), [False, False, False, False, True, True, False])
    assert not TH.prior_fixed([3, 2], [2, 1]).any()


def test_fit_recovers_the_generating_parameters_from_exact_records():
    rng = np.random.default_rng(5)
    for _ in range(10):
        true = THETA * np.exp(0.4 * rng.standard_normal(7))
        true[TH.GAMMA] = rng.uniform(1.2, 6.0)
        K, nodes, m, s, T = records(true, 60, 16, rng)
        theta, f, _ = TH.fit(K, nodes, m, s, T, n_starts=3)          # one start alone can end in a local minimum
        assert f < 1e-8
        pred = TH.t_iter(theta, K, nodes, m, s)[0]
        assert np.max(np.abs(pred / T - 1.0)) < 1e-6
        assert np.all(theta[:6] >= 0.0) and 1.0 <= theta[TH.GAMMA] <= 10.0


def test_fit_of_noisy_records_reaches_the_noise_level_and_a_stationary_point():
    rng = np.random.default_rng(6)
    K, nodes, m, s, T = records(THETA, 200, 16, rng, sigma=0.03)
    theta, f, res = TH.fit(K, nodes, m, s, T)
    assert 0.02 < f < 0.035 and f <= TH.rmsle(THETA, K, nodes, m, s, T) + 1e-12
    _, g = TH.rmsle_and_gradient(theta, K, nodes, m, s, T)
    lo = np.array([0.0] * 6 + [1.0])
    hi = np.array([np.inf] * 6 + [10.0])
    free = ~(((theta <= lo) & (g > 0)) | ((theta >= hi) & (g < 0)))
    assert np.max(np.abs(g[free] * np.maximum(theta[free], 1e-3))) < 1e-6   # scaled projected gradient


def test_generated_records_are_well_formed():
    ob = W.observations("physical")
    n = ob["count"]
    assert n.min() >= 6 and n.max() <= ob["K"].shape[1]
    for j in range(ob["K"].shape[0]):
        k, nd = ob["K"][j, :n[j]], ob["nodes"][j, :n[j]]
        assert np.all(k >= 1) and np.all(nd >= 1) and np.all(nd <= k) and np.all(ob["T"][j, :n[j]] > 0)
    again = W.observations("physical")
    assert all(np.array_equal(ob[key], again[key]) for key in ob)


def test_more_starting_points_never_make_the_fit_worse():
    ob = W.observations("physical")
    for j in range(0, 30, 3):
        n = ob["count"][j]
        r = tuple(ob[k][j, :n] for k in ("K", "nodes", "m", "s", "T"))
        f1, f3, f5 = (TH.fit(*r, n_starts=k)[1] for k in (1, 3, 5))
        assert f5 <= f3 <= f1
