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
