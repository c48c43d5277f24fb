"""Pins for SPEEDUP / FITNESS_p, the re-allocation penalty and the constraint
check of the CPU checker (Sec. 4.2 of the paper).  No GPU needed."""
import os

import numpy as np
import pytest

import oracle as O
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def run(wl, population=None, p=None, flags=0, current=None, delta=None):
    c = wl.cfg
    return O.fitness(wl.population if population is None else population, wl.job_params, wl.m_grid,
                     wl.fair_share, wl.current_alloc if current is None else current, wl.node_capacity,
                     c.p if p is None else p, c.delta if delta is None else delta, c.Gs, flags)


# ------------------------------------------------------------ Eq. 14

def test_pmean_golden_closed_forms():
    S = [1.0, 2.0, 0.5, 4.0]
    with open(os.path.join(GOLDEN, "pmean_vectors.txt")) as f:
        rows = [l.split("#")[0].split() for l in f if l.split("#")[0].strip()]
    assert len(rows) == 5
    for p, want in rows:
        assert O.pmean(S, None, float(p)) == pytest.approx(float(want), rel=1e-11)


def test_pmean_special_orders():
    rng = np.random.default_rng(7)
    S = rng.uniform(0.2, 5.0, 37)
    assert O.pmean(S, None, 1.0) == pytest.approx(S.mean(), rel=1e-14)                 # arithmetic
    assert O.pmean(S, None, -1.0) == pytest.approx(len(S) / (1.0 / S).sum(), rel=1e-14)  # harmonic
    assert O.pmean(S, None, 0.0) == pytest.approx(np.exp(np.log(S).mean()), rel=1e-14)   # geometric
    assert O.pmean(S, None, 2.0) == pytest.approx(np.sqrt((S ** 2).mean()), rel=1e-14)
    assert O.pmean(S, None, -300.0) == pytest.approx(S.min(), rel=2e-2)                # p -> -inf: minimum
    assert O.pmean(S, None, -300.0) >= S.min()


def test_pmean_monotone_in_p_and_bounded():
    rng = np.random.default_rng(8)
    for _ in range(50):
        S = rng.uniform(0.1, 10.0, int(rng.integers(2, 40)))
        ps = [-20, -5, -1, -0.3, 0.0, 0.5, 1.0, 3.0, 20.0]
        v = [O.pmean(S, None, p) for p in ps]
        assert all(b >= a * (1 - 1e-13) for a, b in zip(v, v[1:]))
        assert S.min() * (1 - 1e-13) <= v[0] and v[-1] <= S.max() * (1 + 1e-13)


def test_pmean_weights():
    S = np.array([1.0, 4.0])
    assert O.pmean(S, [3.0, 1.0], 1.0) == pytest.approx(1.75)
    assert O.pmean(S, [1.0, 0.0], -1.0) == 1.0
    # integer weights equal repetition
    assert O.pmean(S, [2.0, 3.0], -1.0) == pytest.approx(O.pmean([1.0, 1.0, 4.0, 4.0, 4.0], None, -1.0), rel=1e-15)


def test_pmean_with_a_zero_speedup():
    S = [2.0, 0.0, 3.0]
    assert O.pmean(S, None, -1.0) == 0.0       # 0^-1 = inf, inf^-1 = 0
    assert O.pmean(S, None, 0.0) == 0.0        # geometric mean with a zero factor
    assert O.pmean(S, None, 1.0) == pytest.approx(5.0 / 3.0)


# ------------------------------------------------------------ restart factor

def test_realloc_factor():
    assert O.realloc_factor(3600.0, 2.0, 30.0) == pytest.approx(3540.0 / 3630.0, rel=1e-16)
    assert O.realloc_factor(3600.0, 2.0, 30.0) == pytest.approx(0.975206611570, rel=1e-11)
    assert O.realloc_factor(500.0, 0.0, 30.0) == 500.0 / 530.0
    assert O.realloc_factor(500.0, 7.0, 0.0) == 1.0
    f = [O.realloc_factor(5000.0, R, 30.0) for R in range(6)]
    assert all(a > b for a, b in zip(f, f[1:])) and f[0] < 1.0


# ------------------------------------------------------------ Eq. 15 and the whole call

@pytest.mark.parametrize("name", ["tiny", "physical"])
@pytest.mark.parametrize("p", [-10.0, -1.0, 0.0, 0.5, 1.0])
def test_fair_share_allocation_has_fitness_exactly_one(name, p):
    wl = W.make(name, current="fair")
    r = run(wl, population=wl.population[:1], p=p)
    assert np.array_equal(wl.population[0], wl.current_alloc)
    assert r["status"] == 0 and r["violations"][0] == 0
    assert np.all(r["speedup"][0] == 1.0)
    assert r["fitness"][0] == 1.0


def test_speedup_is_ratio_to_fair_share_goodput_and_penalty_applies_to_changed_rows():
    wl = W.make("tiny")
    c = wl.cfg
    r = run(wl)
    r0 = run(wl, flags=O.FLAG_NO_PENALTY)
    K = wl.population.sum(2)
    nodes = (wl.population > 0).sum(2)
    changed = (wl.population != wl.current_alloc[None]).any(2)
    running = wl.current_alloc.sum(1) > 0
    for cand in range(c.P):
        for j in range(c.J):
            jb = O.job_from_params(wl.job_params, j)
            g, im, is_ = O.best_goodput(jb, wl.m_grid[j], c.Gs, int(K[cand, j]), int(nodes[cand, j]))
            d, _, _ = O.best_goodput(jb, wl.m_grid[j], c.Gs, int(wl.fair_share[j, 0]), int(wl.fair_share[j, 1]))
            assert r["best_goodput"][cand, j] == g
            assert r["best_m"][cand, j] == (wl.m_grid[j, im] if im >= 0 else -1)
            assert r["best_s"][cand, j] == is_
            assert r0["speedup"][cand, j] == g / d
            f = O.realloc_factor(wl.param("age_T")[j], wl.param("restarts_R")[j], c.delta)
            want = g / d * f if (changed[cand, j] and running[j]) else g / d
            assert r["speedup"][cand, j] == want
    assert changed.any() and (~changed).any()


def test_pending_job_is_not_penalised_and_zero_gpus_give_zero_speedup():
    wl = W.make("tiny")
    cur = wl.current_alloc.copy()
    cur[3] = 0                                         # job 3 is pending: nothing to restart
    r = run(wl, current=cur)
    r0 = run(wl, current=cur, flags=O.FLAG_NO_PENALTY)
    assert np.array_equal(r["speedup"][:, 3], r0["speedup"][:, 3])
    pop = wl.population.copy()
    pop[:, 5, :] = 0                                   # job 5 gets nothing anywhere
    r = run(wl, population=pop)
    assert np.all(r["speedup"][:, 5] == 0.0) and np.all(r["best_m"][:, 5] == -1) and np.all(r["best_s"][:, 5] == -1)
    ok = r["violations"] == 0
    assert np.all(r["fitness"][ok] == 0.0)             # p = -1: one starved job zeroes the harmonic mean
    r1 = run(wl, population=pop, p=1.0)
    assert np.all(r1["fitness"][ok] > 0.0)


def test_fitness_is_the_pmean_of_the_speedups():
    wl = W.make("physical")
    for p in (-1.0, 0.0, 0.5, 1.0):
        r = run(wl, p=p)
        for cand in range(wl.cfg.P):
            if r["violations"][cand] == 0:
                assert r["fitness"][cand] == O.pmean(r["speedup"][cand], wl.param("weight"), p)
            else:
                assert r["fitness"][cand] == -float(r["violations"][cand])


def test_constraint_check_counts_capacity_and_interference():
    cfg = W.custom("hand", P=1, J=3, N=3, cap=4, Gm=4, Gs=2)
    wl = W.make(cfg, current="fair")
    A = np.zeros((1, 3, 3), np.int32)
    A[0, 0] = [2, 2, 0]        # distributed on nodes 0, 1
    A[0, 1] = [0, 1, 1]        # distributed on nodes 1, 2 -> shares node 1 with job 0: one violation
    A[0, 2] = [3, 0, 0]        # single node; node 0 holds 5 > 4: one GPU over capacity
    r = run(wl, population=A)
    assert r["violations"][0] == 2 and r["fitness"][0] == -2.0
    r2 = run(wl, population=A, flags=O.FLAG_NO_CHECK)
    assert r2["violations"][0] == 2 and r2["fitness"][0] > 0.0
    A[0, 2] = [2, 0, 0]
    assert run(wl, population=A)["violations"][0] == 1
    A[0, 1] = [0, 0, 2]
    r = run(wl, population=A)
    assert r["violations"][0] == 0 and r["fitness"][0] > 0.0


def test_generated_populations_are_feasible_except_the_spoiled_slice():
    for name in ("tiny", "physical", "mid"):
        wl = W.make(name)
        r = run(wl)
        bad = np.flatnonzero(r["violations"] > 0)
        assert set(bad) <= {i for i in range(wl.cfg.P) if i % 20 == 7}
        assert r["status"] == 0
        assert np.all(r["fitness"][bad] < 0)
        good = r["violations"] == 0
        assert np.all(r["fitness"][good] >= 0)
        assert (r["fitness"][good] > 0).mean() > 0.7


def test_status_word():
    wl = W.make("tiny")
    jp = wl.job_params.copy()
    jp[W.PARAM_INDEX["gamma"], 2] = 0.5
    r = O.fitness(wl.population, jp, wl.m_grid, wl.fair_share, wl.current_alloc, wl.node_capacity, -1.0, 30.0, wl.cfg.Gs)
    assert r["status"] & O.ST_BAD_PARAM
    jp = wl.job_params.copy()
    jp[W.PARAM_INDEX["age_T"], 1] = 10.0
    jp[W.PARAM_INDEX["restarts_R"], 1] = 3.0
    r = O.fitness(wl.population, jp, wl.m_grid, wl.fair_share, wl.current_alloc, wl.node_capacity, -1.0, 30.0, wl.cfg.Gs)
    assert r["status"] == O.ST_BAD_RESTART
    jp = wl.job_params.copy()
    jp[W.PARAM_INDEX["M0"], 0] = 1e9
    jp[W.PARAM_INDEX["M_max"], 0] = 2e9
    r = O.fitness(wl.population, jp, wl.m_grid, wl.fair_share, wl.current_alloc, wl.node_capacity, -1.0, 30.0, wl.cfg.Gs)
    assert r["status"] == O.ST_ZERO_FAIR and np.all(r["speedup"][:, 0] == 0.0)
    pop = wl.population.copy()
    pop[2, 2, 1] = -1
    r = O.fitness(pop, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc, wl.node_capacity, -1.0, 30.0, wl.cfg.Gs)
    assert r["status"] == O.ST_NEG_ALLOC


def test_invalid_arguments_are_rejected():
    wl = W.make("tiny")
    with pytest.raises(ValueError):
        O.fitness(wl.population, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc, wl.node_capacity,
                  float("nan"), 30.0, wl.cfg.Gs)
    with pytest.raises(ValueError):
        O.fitness(wl.population, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc, wl.node_capacity,
                  -1.0, -5.0, wl.cfg.Gs)


def test_more_gpus_never_reduce_the_best_goodput_of_a_single_node_job():
    # max over (m,s) of goodput with K GPUs on one node vs K = 1: adding GPUs on the same node can only
    # help while T_sync stays small; checked here in the regime alpha_sync_local = beta_sync_local = 0
    # (the paper's exploration prior: throughput assumed to scale perfectly)
    jb = O.job(0.1, 0.001, 0.0, 0.0, 0.2, 0.02, 2.0, 1e4, 32.0, 1024.0)
    grid = W.m_grid(np.array([256]), 32)[0]
    g = [O.best_goodput(jb, grid, 8, K, 1)[0] for K in range(1, 5)]
    assert all(b >= a for a, b in zip(g, g[1:]))
