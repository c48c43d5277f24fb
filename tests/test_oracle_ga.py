"""Pins for the counter-based generator and the population-search step of the
CPU checker (Sec. 4.3 of the paper gives only the outline, so the operators are
pinned by their invariants).  No GPU needed."""
import os

import numpy as np
import pytest

import oracle as O
import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
SEED = 0x1234_5678_9ABC_DEF0


def constraint_violations(A, cap):
    """Per candidate: GPUs over capacity + extra multi-node jobs per node (numpy, independent of the oracle)."""
    col = A.sum(1)
    over = np.clip(col - cap[None, :], 0, None).sum(1)
    dist = (A > 0).sum(2) >= 2
    dn = ((A > 0) & dist[:, :, None]).sum(1)
    return over + np.clip(dn - 1, 0, None).sum(1)


def test_philox_known_answers():
    n = 0
    with open(os.path.join(GOLDEN, "philox_kat.txt")) as f:
        for line in f:
            line = line.split("#")[0].split()
            if not line:
                continue
            w = [int(x, 16) for x in line]
            assert list(O.philox4x32_10(w[0:4], w[4:6])) == w[6:10]
            n += 1
    assert n == 3


def test_philox_is_a_bijection_of_the_counter_on_a_sample():
    outs = {tuple(O.philox4x32_10([i, 0, 0, 0], [7, 9])) for i in range(2000)}
    assert len(outs) == 2000
    # word 0 is roughly uniform: mean of 2000 draws within 5 sigma of 2^31
    w0 = np.array([o[0] for o in outs], dtype=np.float64)
    assert abs(w0.mean() - 2.0 ** 31) < 5 * (2.0 ** 32 / np.sqrt(12 * 2000))


def test_rank_orders_by_fitness_then_index():
    rng = np.random.default_rng(11)
    f = rng.choice([0.0, 0.5, 0.7, -3.0, 1.25], 200)
    f[17] = np.nan
    order = O.rank(f)
    key = np.where(np.isnan(f), -np.inf, f)
    want = np.lexsort((np.arange(f.size), -key))
    assert np.array_equal(order, want)
    assert order[-1] == 17 or key[order[-1]] == -np.inf


def test_repair_postconditions_and_only_removals():
    rng = np.random.default_rng(12)
    for trial in range(60):
        J, N = int(rng.integers(1, 12)), int(rng.integers(1, 9))
        cap = rng.integers(1, 6, N).astype(np.int32)
        A = rng.integers(0, 4, (J, N)).astype(np.int32) * (rng.uniform(size=(J, N)) < 0.6)
        A = A.astype(np.int32)
        B = O.repair(A, cap, SEED, trial, 5)
        assert np.all(B >= 0) and np.all(B <= A)
        assert constraint_violations(B[None], cap)[0] == 0
        # a feasible matrix is left alone
        assert np.array_equal(O.repair(B, cap, SEED, trial + 1, 9), B)


def test_repair_capacity_removes_exactly_the_excess_in_cyclic_order():
    cap = np.array([4], dtype=np.int32)
    A = np.array([[3], [2], [0], [4]], dtype=np.int32)        # 9 GPUs asked on a 4-GPU node
    B = O.repair(A, cap, SEED, 3, 8)
    assert B.sum() == 4
    r = O.philox4x32_10([3, 8, 0, 4], [SEED & 0xFFFFFFFF, SEED >> 32])
    j0 = (int(r[0]) * 4) >> 32
    want = A[:, 0].copy()
    excess = 5
    for t in range(4):
        j = (j0 + t) % 4
        take = min(want[j], excess)
        want[j] -= take
        excess -= take
    assert np.array_equal(B[:, 0], want)


def test_repair_interference_keeps_the_largest_holder():
    cap = np.full(3, 8, dtype=np.int32)
    A = np.array([[1, 2, 0],      # multi-node, 2 GPUs on node 1
                  [0, 3, 1],      # multi-node, 3 GPUs on node 1 -> kept there
                  [0, 2, 0]],     # single node: never affected
                 dtype=np.int32)
    B = O.repair(A, cap, SEED, 0, 0)
    assert np.array_equal(B, [[1, 0, 0], [0, 3, 1], [0, 2, 0]])
    # tie on the GPU count: lowest job index stays
    A = np.array([[1, 2, 0], [0, 2, 1]], dtype=np.int32)
    B = O.repair(A, cap, SEED, 0, 0)
    assert np.array_equal(B, [[1, 2, 0], [0, 0, 1]])


def step(wl, parents, fit, gen, elite=None, mut=1 << 29):
    P = parents.shape[0]
    return O.ga_step(parents, fit, wl.node_capacity, SEED, gen, P // 2 if elite is None else elite, mut)


def test_ga_step_elites_are_copied_in_rank_order_and_children_are_feasible():
    wl = W.make("physical")
    c = wl.cfg
    fit = O.fitness(wl.population, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc,
                    wl.node_capacity, c.p, c.delta, c.Gs)["fitness"]
    kids = step(wl, wl.population, fit, 0)
    order = O.rank(fit)
    for k in range(c.P // 2):
        assert np.array_equal(kids[k], wl.population[order[k]])
    assert np.all(kids >= 0)
    assert np.all(constraint_violations(kids[c.P // 2:], wl.node_capacity) == 0)
    assert not np.array_equal(kids[c.P // 2:], wl.population[c.P // 2:])


def test_ga_step_without_mutation_takes_every_row_from_one_of_two_survivors():
    wl = W.make("tiny")
    c = wl.cfg
    fit = np.arange(c.P, dtype=np.float64)[::-1].copy()       # candidate 0 best
    good = constraint_violations(wl.population, wl.node_capacity) == 0
    fit[~good] = -1.0
    elite = 4
    kids = step(wl, wl.population, fit, 2, elite=elite, mut=0)
    order = O.rank(fit)
    surv = wl.population[order[:elite]]
    for ch in kids[elite:]:
        # before repair each row equals some survivor's row; repair only removes GPUs
        for j in range(c.J):
            assert any(np.all(ch[j] <= s[j]) for s in surv)
    # parents are drawn by word 0 and 1 of the "parent" counter block
    for cidx in range(elite, c.P):
        r = O.philox4x32_10([2, cidx, 0, 0], [SEED & 0xFFFFFFFF, SEED >> 32])
        a, b = order[(int(r[0]) * elite) >> 32], order[(int(r[1]) * elite) >> 32]
        if int(r[2]) & 1:
            b = a                                  # a child of one parent
        for j in range(c.J):
            bit = int(O.philox4x32_10([2, cidx, j, 1], [SEED & 0xFFFFFFFF, SEED >> 32])[0]) & 1
            src = wl.population[b if bit else a][j]
            assert np.all(kids[cidx][j] <= src)


def test_ga_step_is_deterministic_and_resumable():
    wl = W.make("tiny")
    c = wl.cfg

    def fitness_of(pop):
        return O.fitness(pop, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc, wl.node_capacity,
                         c.p, c.delta, c.Gs)["fitness"]

    pop = wl.population
    history = []
    for g in range(6):
        pop = step(wl, pop, fitness_of(pop), g)
        history.append(pop)
    # same inputs twice -> identical output
    assert np.array_equal(step(wl, history[2], fitness_of(history[2]), 3), history[3])
    # the state is (population, seed, generation): restarting at generation 4 continues identically
    pop = history[3]
    for g in range(4, 6):
        pop = step(wl, pop, fitness_of(pop), g)
    assert np.array_equal(pop, history[5])
    # a different generation number gives different children
    assert not np.array_equal(step(wl, history[2], fitness_of(history[2]), 4), history[3])


def test_ga_search_improves_the_best_fitness():
    wl = W.make("physical", current="fair")
    c = wl.cfg

    def fitness_of(pop):
        return O.fitness(pop, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc, wl.node_capacity,
                         c.p, c.delta, c.Gs)["fitness"]

    pop = wl.population
    best0 = fitness_of(pop).max()
    best = best0
    for g in range(30):
        f = fitness_of(pop)
        assert f.max() >= best - 1e-15          # elitism: the best candidate is never lost
        best = f.max()
        pop = step(wl, pop, f, g)
    assert best >= 1.0                           # candidate 0 (fair share, unchanged) scores exactly 1
    assert fitness_of(pop).max() >= best0


def test_mutation_moves():
    # one job, several nodes, mutation certain: the child differs from the parent by exactly one move
    parents = np.zeros((8, 1, 5), np.int32)
    parents[:, 0, :] = [2, 0, 1, 0, 0]          # occupies nodes 0 and 2
    cap = np.full(5, 8, np.int32)
    fit = np.ones(8)
    seen = set()
    for gen in range(40):
        kids = O.ga_step(parents, fit, cap, SEED, gen, 1, 0xFFFFFFFF)
        for cidx in range(1, 8):
            r = O.philox4x32_10([gen, cidx, 0, 3], [SEED & 0xFFFFFFFF, SEED >> 32])
            move, x = int(r[0]) % 3, int(r[1])
            want = np.array([2, 0, 1, 0, 0])
            if move == 2:
                want[:] = 0
                want[(x * 5) >> 32] = 3
            else:
                n = [0, 2][(x * 2) >> 32]       # the drawn one of the two occupied nodes
                want[n] += 1 if move == 0 else -1
            # single job: interference repair cannot trigger, capacity 8 never exceeded
            assert np.array_equal(kids[cidx, 0], want)
            seen.add(move)
    assert seen == {0, 1, 2}
    # a job without GPUs: grow starts it on a drawn node, shrink leaves it alone
    parents[:] = 0
    for gen in range(20):
        kids = O.ga_step(parents, fit, cap, SEED, gen, 1, 0xFFFFFFFF)
        for cidx in range(1, 8):
            r = O.philox4x32_10([gen, cidx, 0, 3], [SEED & 0xFFFFFFFF, SEED >> 32])
            move, x = int(r[0]) % 3, int(r[1])
            want = np.zeros(5, np.int64)
            if move == 0:
                want[(x * 5) >> 32] = 1
            assert np.array_equal(kids[cidx, 0], want)


def test_search_finds_better_allocations_than_the_fair_share():
    """With spare GPUs in the cluster (64 GPUs, 30 jobs at 2 each) and about one mutation per child, the search
    must beat candidate 0, which keeps every job at its fair share and scores exactly 1."""
    wl = W.make("physical", current="fair")
    c = wl.cfg

    def fitness_of(pop):
        return O.fitness(pop, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc, wl.node_capacity,
                         c.p, c.delta, c.Gs)["fitness"]

    pop = wl.population
    assert fitness_of(pop).max() == 1.0
    for g in range(40):
        pop = O.ga_step(pop, fitness_of(pop), wl.node_capacity, SEED, g, c.P // 2, (1 << 32) // c.J)
    f = fitness_of(pop)
    assert f.max() > 1.01
    assert np.all(constraint_violations(pop[np.argsort(-f)[:10]], wl.node_capacity) == 0)


def test_in_place_step_is_the_out_of_place_step_with_children_in_the_slots_of_the_losers():
    wl = W.make("physical")
    c = wl.cfg
    rng = np.random.default_rng(12)
    fit = rng.uniform(0.1, 1.0, c.P)
    fit[3] = fit[40] = fit[77]
    order = O.rank(fit)
    for elite in (1, c.P // 2, c.P):
        out = O.ga_step(wl.population, fit, wl.node_capacity, 77, 2, elite, 1 << 29)
        inp = O.ga_step(wl.population, fit, wl.node_capacity, 77, 2, elite, 1 << 29, flags=O.GA_IN_PLACE)
        assert np.array_equal(inp[order], out)                                  # child c sits in slot order[c]
        assert np.array_equal(inp[order[:elite]], wl.population[order[:elite]])  # survivors did not move


def test_gpu_limit_on_a_row_keeps_gpus_in_ascending_node_order():
    assert O.cap_row([3, 0, 2, 4], 4).tolist() == [3, 0, 1, 0]
    assert O.cap_row([3, 0, 2, 4], 5).tolist() == [3, 0, 2, 0]
    assert O.cap_row([3, 0, 2, 4], 9).tolist() == [3, 0, 2, 4]
    assert O.cap_row([3, 0, 2, 4], 0).tolist() == [0, 0, 0, 0]
    assert O.cap_row([3, 0, 2, 4], -5).tolist() == [0, 0, 0, 0]
    assert O.cap_row([0, 0, 7], 2).tolist() == [0, 0, 2]
    rng = np.random.default_rng(5)
    for _ in range(200):
        row = rng.integers(0, 5, 12).astype(np.int32) * (rng.uniform(size=12) < 0.4)
        cap = int(rng.integers(0, 20))
        got = O.cap_row(row, cap)
        assert got.sum() == min(cap, row.sum()) and np.all(got <= row) and np.all(got >= 0)
        nz = np.flatnonzero(got != row)                      # everything before the first cut is intact
        if nz.size:
            assert np.all(got[nz[0] + 1:] == 0)


def test_ga_step_with_job_gpu_limits():
    wl = W.make("physical")
    c = wl.cfg
    fit = np.linspace(1.0, 0.1, c.P)
    base = O.ga_step(wl.population, fit, wl.node_capacity, 5, 1, c.P // 2, 1 << 30)
    # a limit nobody reaches changes nothing
    same = O.ga_step(wl.population, fit, wl.node_capacity, 5, 1, c.P // 2, 1 << 30, job_gpu_cap=np.full(c.J, 10**6, np.int32))
    assert np.array_equal(base, same)
    limits = np.random.default_rng(6).integers(0, 4, c.J).astype(np.int32)
    capped = O.ga_step(wl.population, fit, wl.node_capacity, 5, 1, c.P // 2, 1 << 30, job_gpu_cap=limits)
    assert (wl.population.sum(2) > limits[None]).any()                     # the parents do break the limits
    assert np.all(capped[c.P // 2:].sum(2) <= limits[None])                # no child does
    assert np.array_equal(capped[:c.P // 2], base[:c.P // 2])              # survivors are kept as they are
    assert np.all(capped >= 0)
