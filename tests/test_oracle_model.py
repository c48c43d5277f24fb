"""Pins for the goodput model of the CPU checker (no GPU needed).

Each test ties one piece of oracle/pollux_ref.c to something the paper or plain
mathematics fixes: closed forms, limits, hand-derived values, brute force.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")

# the parameter set of tests/golden/goodput_vectors.txt
HAND = dict(alpha_g=0.1, beta_g=0.001, alpha_sl=0.05, beta_sl=0.01, alpha_sn=0.2, beta_sn=0.02,
            phi=1000.0, M0=100.0, Mmax=3200.0)


def hand_job(gamma):
    return O.job(gamma=gamma, **HAND)


def read_vectors(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                rows.append(line)
    return rows


# ------------------------------------------------------------ Eq. 6 efficiency

def test_efficiency_is_one_at_initial_batch_size():
    rng = np.random.default_rng(1)
    for _ in range(200):
        phi, M0 = float(rng.uniform(1, 1e6)), float(rng.integers(1, 4096))
        assert O.efficiency(phi, M0, M0) == 1.0


def test_efficiency_is_a_fraction_and_decreasing_above_M0():
    rng = np.random.default_rng(2)
    for _ in range(200):
        phi, M0 = float(rng.uniform(1, 1e6)), float(rng.integers(1, 4096))
        Ms = M0 * np.array([1, 1.5, 2, 8, 32])
        e = [O.efficiency(phi, M0, float(M)) for M in Ms]
        assert all(0.0 < x <= 1.0 for x in e)
        assert all(a > b for a, b in zip(e, e[1:]))


def test_efficiency_exact_rational_value():
    # (1000 + 100) / (1000 + 200) = 11/12
    assert O.efficiency(1000.0, 100.0, 200.0) == pytest.approx(float(Fraction(11, 12)), rel=1e-16)
    # phi -> infinity: every batch size is perfectly efficient; phi -> 0: efficiency M0/M
    assert O.efficiency(1e300, 64.0, 2048.0) == 1.0
    assert O.efficiency(1e-300, 64.0, 2048.0) == pytest.approx(64.0 / 2048.0, rel=1e-15)


# ------------------------------------------------------------ Eq. 8 / Eq. 9

def test_tgrad_linear():
    assert O.tgrad(0.1, 0.001, 100.0) == 0.1 + 0.001 * 100.0
    assert O.tgrad(0.25, 0.0, 12345.0) == 0.25
    assert O.tgrad(0.0, 0.5, 4.0) == 2.0


def test_tsync_cases_on_all_placements_of_a_2x2_cluster():
    jb = hand_job(2.0)
    for a0, a1 in itertools.product(range(3), range(3)):
        K, nodes = a0 + a1, (a0 > 0) + (a1 > 0)
        t = O.tsync(jb, K, nodes)
        if K <= 1:
            assert t == 0.0
        elif nodes == 1:
            assert t == 0.05 + 0.01 * (K - 2)
        else:
            assert t == 0.2 + 0.02 * (K - 2)
    # two GPUs: only the constant term; the retrogression term starts at the third GPU
    assert O.tsync(jb, 2, 1) == 0.05 and O.tsync(jb, 2, 2) == 0.2
    assert O.tsync(jb, 3, 1) == pytest.approx(0.06) and O.tsync(jb, 3, 2) == pytest.approx(0.22)
    assert O.tsync(jb, 3, 3) == O.tsync(jb, 3, 2)      # more than two nodes: same pair of parameters


# ------------------------------------------------------------ Eq. 10 / Eq. 11

def test_overlap_gamma_one_is_the_plain_sum_and_zero_sync_leaves_tgrad():
    assert O.titer(0.2, 0.05, 1.0, 0) == 0.2 + 0.05
    assert O.titer(0.2, 0.0, 3.7, 0) == 0.2
    assert O.titer(0.2, 0.0, 3.7, 5) == 5 * 0.2 + 0.2


def test_overlap_between_max_and_sum_and_non_increasing_in_gamma():
    rng = np.random.default_rng(3)
    for _ in range(300):
        tg, ts = float(rng.uniform(1e-3, 1.0)), float(rng.uniform(1e-3, 1.0))
        gammas = [1.0, 1.3, 2.0, 3.0, 5.0, 10.0]
        vals = [O.titer(tg, ts, g, 0) for g in gammas]
        for v in vals:
            assert max(tg, ts) * (1 - 1e-15) <= v <= (tg + ts) * (1 + 1e-15)
        assert all(a >= b * (1 - 1e-15) for a, b in zip(vals, vals[1:]))
        assert vals[-1] <= max(tg, ts) * 2 ** 0.1 * (1 + 1e-15)     # gamma = 10 is within 2^(1/10) of the max


def test_overlap_closed_forms_square_and_cube():
    # gamma = 2: Euclidean norm; 3-4-5 triangle scaled by 0.1
    assert O.titer(0.3, 0.4, 2.0, 0) == pytest.approx(0.5, rel=1e-15)
    # gamma = 3: cube root of 0.1^3 + 0.2^3 = 0.009
    assert O.titer(0.1, 0.2, 3.0, 0) == pytest.approx(0.009 ** (1.0 / 3.0), rel=1e-15)
    # equal terms: (2 t^g)^(1/g) = t * 2^(1/g)
    assert O.titer(0.25, 0.25, 4.0, 0) == pytest.approx(0.25 * 2 ** 0.25, rel=1e-15)


def test_accumulation_adds_s_unsynchronised_passes():
    tg, ts, g = 0.15, 0.24, 3.0
    last = O.titer(tg, ts, g, 0)
    for s in range(0, 12):
        assert O.titer(tg, ts, g, s) == s * tg + last


def test_throughput_monotone_in_s_and_flat_without_sync():
    # THROUGHPUT = K m (s+1) / (s Tg + last) with last >= Tg: non-decreasing in s, -> K m / Tg
    jb = O.job(0.1, 0.001, 0.05, 0.01, 0.2, 0.02, 2.5, 1e300, 1.0, 1e18)   # efficiency == 1: goodput = throughput
    K, nodes, m = 4, 2, 64
    thr = [O.goodput(jb, K, nodes, m, s)[0] for s in range(64)]
    assert all(b >= a for a, b in zip(thr, thr[1:]))
    limit = K * m / O.tgrad(0.1, 0.001, m)
    assert thr[-1] < limit and O.goodput(jb, K, nodes, m, 100000)[0] == pytest.approx(limit, rel=1e-4)
    # one GPU: no synchronisation, throughput independent of s
    one = [O.goodput(jb, 1, 1, m, s)[0] for s in range(16)]
    assert np.allclose(one, m / O.tgrad(0.1, 0.001, m), rtol=1e-15)


# ------------------------------------------------------------ hand-derived vectors

def test_hand_derived_goodput_vectors():
    for row in read_vectors("goodput_vectors.txt"):
        left, right = row.split("|")
        K, nodes, m, s, gamma = [float(x) for x in left.split()]
        ts, last, t_iter, M, eff, good = [float(x) for x in right.split()]
        jb = hand_job(gamma)
        K, nodes, m, s = int(K), int(nodes), int(m), int(s)
        assert O.tsync(jb, K, nodes) == pytest.approx(ts, rel=1e-12, abs=0)
        tg = O.tgrad(HAND["alpha_g"], HAND["beta_g"], m)
        assert O.titer(tg, O.tsync(jb, K, nodes), gamma, 0) == pytest.approx(last, rel=1e-11)
        assert O.titer(tg, O.tsync(jb, K, nodes), gamma, s) == pytest.approx(t_iter, rel=1e-11)
        assert K * m * (s + 1) == M
        assert O.efficiency(HAND["phi"], HAND["M0"], M) == pytest.approx(eff, rel=1e-11)
        g, ok = O.goodput(jb, K, nodes, m, s)
        assert ok and g == pytest.approx(good, rel=1e-9)


def test_goodput_equals_throughput_iff_efficiency_is_perfect():
    jb = hand_job(2.0)
    g, ok = O.goodput(jb, 1, 1, 100, 0)      # M = M0 = 100: efficiency 1
    assert ok and g == 100.0 / 0.2
    g2, ok2 = O.goodput(jb, 2, 1, 100, 0)    # M = 200 > M0: strictly below throughput
    assert ok2 and g2 < 200.0 / O.titer(0.2, 0.05, 2.0, 0)


def test_feasibility_limits():
    jb = hand_job(2.0)                        # M0 = 100, M_max = 3200
    assert O.goodput(jb, 1, 1, 99, 0) == (0.0, False)        # M < M0
    assert O.goodput(jb, 1, 1, 100, 0)[1]                    # M = M0 allowed
    assert O.goodput(jb, 4, 1, 100, 7)[1]                    # M = 3200 = M_max allowed
    assert O.goodput(jb, 4, 1, 100, 8) == (0.0, False)       # M = 3600 > M_max
    assert O.goodput(jb, 0, 0, 100, 0) == (0.0, False)       # no GPUs


# ------------------------------------------------------------ Eq. 13 argmax

def brute_goodput(p, K, nodes, m, s):
    """Eq. 4-11 typed out independently (plain Python floats)."""
    M = K * m * (s + 1)
    if K <= 0 or M < p["M0"] or M > p["Mmax"]:
        return None
    tg = p["alpha_g"] + p["beta_g"] * m
    if K == 1:
        ts = 0.0
    elif nodes == 1:
        ts = p["alpha_sl"] + p["beta_sl"] * (K - 2)
    else:
        ts = p["alpha_sn"] + p["beta_sn"] * (K - 2)
    if ts == 0.0:
        last = tg
    elif p["gamma"] == 1.0:
        last = tg + ts
    else:
        last = (tg ** p["gamma"] + ts ** p["gamma"]) ** (1.0 / p["gamma"])
    return (M / (s * tg + last)) * ((p["phi"] + p["M0"]) / (p["phi"] + M))


def test_argmax_against_brute_force_on_tiny_grids():
    rng = np.random.default_rng(5)
    names = ["alpha_g", "beta_g", "alpha_sl", "beta_sl", "alpha_sn", "beta_sn", "gamma", "phi", "M0", "Mmax"]
    for trial in range(400):
        p = dict(alpha_g=rng.uniform(0.01, 0.2), beta_g=math.exp(rng.uniform(math.log(1e-5), math.log(1e-3))),
                 alpha_sl=rng.uniform(0.005, 0.05), beta_sl=rng.uniform(0.001, 0.01),
                 alpha_sn=rng.uniform(0.02, 0.2), beta_sn=rng.uniform(0.005, 0.05),
                 gamma=float(rng.choice([1.0, 1.5, 2.0, 3.3, 10.0])), phi=math.exp(rng.uniform(4, 12)),
                 M0=float(rng.choice([8, 32, 100])))
        p["Mmax"] = p["M0"] * float(rng.choice([1, 2, 32]))
        Gm, Gs = int(rng.integers(1, 5)), int(rng.integers(1, 4))
        grid = np.sort(rng.integers(4, 200, Gm)).astype(np.int32)
        if trial % 3 == 0 and Gm > 1:
            grid[1] = grid[0]                      # duplicated batch size: lowest index must win
        K = int(rng.integers(0, 9))
        nodes = 0 if K == 0 else int(rng.integers(1, min(K, 3) + 1))
        best, bi, bs = 0.0, -1, -1
        for i in range(Gm):
            for s in range(Gs):
                g = brute_goodput(p, K, nodes, int(grid[i]), s)
                if g is not None and g > best:
                    best, bi, bs = g, i, s
        jb = O.job(*[p[n] for n in names])
        g, im, is_ = O.best_goodput(jb, grid, Gs, K, nodes)
        assert (im, is_) == (bi, bs)
        assert g == pytest.approx(best, rel=1e-14)


def test_argmax_ties_go_to_the_lowest_flat_index():
    jb = hand_job(2.0)
    grid = np.array([100, 100, 100], dtype=np.int32)      # three copies of the same batch size
    g, im, is_ = O.best_goodput(jb, grid, 4, 1, 1)
    assert im == 0
    # K = 1: throughput does not depend on s, efficiency falls with M, so s = 0 wins
    assert is_ == 0 and g == 500.0


def test_argmax_nothing_feasible():
    jb = hand_job(2.0)
    assert O.best_goodput(jb, np.array([8, 9], dtype=np.int32), 2, 1, 1) == (0.0, -1, -1)   # M <= 18 < M0
    assert O.best_goodput(jb, np.array([100], dtype=np.int32), 4, 0, 0) == (0.0, -1, -1)    # no GPUs


def test_argmax_gap_reports_distance_to_the_runner_up():
    jb = hand_job(2.0)
    # a single feasible point has no runner-up
    assert O.argmax_gap(jb, np.array([100], dtype=np.int32), 1, 1, 1) == 1.0
    # duplicates of the best value are not runners-up
    grid = np.array([100, 100, 50], dtype=np.int32)
    gap = O.argmax_gap(jb, grid, 2, 2, 1)
    vals = sorted({brute_goodput(dict(HAND, gamma=2.0), 2, 1, int(m), s) for m in grid for s in range(2)} - {None})
    assert gap == pytest.approx((vals[-1] - vals[-2]) / vals[-1], rel=1e-9)


# ------------------------------------------------------------ Sec. 4.3 sampling argmax
def _sampled_brute(jb, m_mem, M_list, s_max, K, nodes):
    """The procedure with nothing closed-form: try s = 0, 1, ... until the per-GPU share fits."""
    best, bm, bs = 0.0, -1, -1
    for M in M_list:
        M = int(M)
        if M <= 0:
            continue
        s = 0
        while -(-M // (K * (s + 1))) > m_mem:
            s += 1
        if s > s_max:
            continue
        m = -(-M // (K * (s + 1)))
        g, ok = O.goodput(jb, K, nodes, m, s)
        if ok and g > best:
            best, bm, bs = g, m, s
    return best, bm, bs


def test_sampling_argmax_against_brute_force():
    rng = np.random.default_rng(43)
    for _ in range(300):
        m_mem = int(rng.integers(1, 200))
        M0 = float(rng.integers(1, 500))
        jb = O.job(rng.uniform(0.01, 0.5), rng.uniform(1e-4, 1e-2), rng.uniform(0, 0.1), rng.uniform(0, 0.02),
                   rng.uniform(0, 0.3), rng.uniform(0, 0.05), rng.uniform(1, 10), rng.uniform(10, 1e5), M0,
                   M0 * rng.uniform(1, 64), float(m_mem))
        K = int(rng.integers(1, 40))
        nodes = 1 if K == 1 else int(rng.integers(1, 5))
        Ms = rng.integers(-2, 20000, int(rng.integers(1, 40))).astype(np.int32)
        s_max = int(rng.integers(0, 20))
        assert O.best_goodput_sampled(jb, Ms, s_max, K, nodes) == _sampled_brute(jb, m_mem, Ms, s_max, K, nodes)


def test_sampling_argmax_points_fit_memory_with_the_fewest_passes():
    rng = np.random.default_rng(44)
    jb = O.job(0.1, 0.001, 0.05, 0.01, 0.2, 0.02, 2.0, 1000.0, 1.0, 1e9, 37.0)
    for _ in range(500):
        K = int(rng.integers(1, 64))
        M = int(rng.integers(1, 100000))
        g, m, s = O.best_goodput_sampled(jb, np.array([M], np.int32), 10**6, K, 2)
        assert g > 0 and 1 <= m <= 37
        assert K * m * (s + 1) >= M > K * (m - 1) * (s + 1)          # m is the ceiling
        assert s == 0 or K * 37 * s < M                               # one pass fewer would not hold M


def test_sampling_argmax_without_a_memory_bound_is_the_dense_argmax_on_one_column():
    """With room for any batch, s = 0 and m = ceil(M/K): the dense routine on that grid with Gs = 1 agrees."""
    rng = np.random.default_rng(45)
    for _ in range(100):
        jb = O.job(0.05, 0.002, 0.03, 0.004, 0.1, 0.01, float(rng.uniform(1, 4)), 5000.0, 64.0, 8192.0, 2.0**31 - 1)
        K = int(rng.integers(1, 33))
        Ms = np.sort(rng.choice(np.arange(64, 8193), 24, replace=False)).astype(np.int32)
        grid = (-(-Ms.astype(np.int64) // K)).astype(np.int32)
        g0, im, is_ = O.best_goodput(jb, grid, 1, K, 2)
        g1, m, s = O.best_goodput_sampled(jb, Ms, 7, K, 2)
        assert g1 == g0 and s == is_ == 0 and m == grid[im]


# ------------------------------------------------------------ non-adaptive jobs (Sec. 4.1: fixed batch size)
def test_a_job_with_a_fixed_batch_size_has_efficiency_one_and_the_fastest_split_wins():
    """M_max = M0 leaves only points with K m (s+1) = M0: Eq. 6 is exactly 1 there, so goodput is throughput
    and the argmax is the split of M0 over GPUs and accumulation passes with the shortest iteration."""
    rng = np.random.default_rng(46)
    grid = np.array([1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128, 192, 256], np.int32)
    for _ in range(200):
        M0 = float(rng.choice([32, 64, 96, 128, 256]))
        jb = O.job(rng.uniform(0.01, 0.2), rng.uniform(1e-5, 1e-3), 0.02, 0.004, 0.1, 0.01, rng.uniform(1, 5),
                   rng.uniform(1e2, 1e5), M0, M0)
        K = int(rng.choice([1, 2, 3, 4, 6, 8, 16]))
        nodes = 1 if K < 4 else 2
        g, im, is_ = O.best_goodput(jb, grid, 8, K, nodes)
        want = 0.0
        for m in grid:
            for s in range(8):
                if K * int(m) * (s + 1) == int(M0):
                    t = O.titer(O.tgrad(jb.alpha_g, jb.beta_g, float(m)), O.tsync(jb, K, nodes), jb.gamma, s)
                    want = max(want, M0 / t)
        if want == 0.0:
            assert g == 0.0 and im == -1
        else:
            assert abs(g - want) <= 1e-15 * want
            assert K * int(grid[im]) * (is_ + 1) == int(M0)
            assert O.efficiency(jb.phi, M0, float(K * int(grid[im]) * (is_ + 1))) == 1.0
