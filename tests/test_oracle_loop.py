"""Pins of the CPU checker for the auto-scaling rule (Sec. 5.3.3) and the simulator tick (Sec. 5.3)."""
import numpy as np

import oracle as O
import oracle.loop as LP
import workloads as W


def test_autoscale_rule_on_tables_worked_out_by_hand():
    # ideal 10 per GPU; per-GPU goodput on 1..5 nodes: 9, 8, 6, 4.9, 3;  U = 2/3 (threshold 6.67), L = 1/2 (5)
    row = np.array([[10.0, 9.0, 8.0, 6.0, 4.9, 3.0]])
    scale = lambda now, table=row, U=2 / 3, L=0.5: int(LP.autoscale(np.repeat(table, 1, 0), [now], U, L)[0])
    assert scale(1) == 3          # 9 > 6.67: add nodes while the next one still predicts >= 5: 8, 6, then 4.9 stops it
    assert scale(2) == 3          # 8 > 6.67
    assert scale(3) == 3          # 6 is not above 6.67: stays
    assert scale(4) == 4 and scale(5) == 5
    assert scale(0) == 0 and scale(6) == 6                         # outside the table: left alone
    assert scale(1, U=0.9) == 1                                    # strict: 9 > 9 is false
    assert scale(1, L=0.0) == 5                                    # nothing stops it but the largest count
    flat = np.array([[10.0, 10.0, 10.0, 10.0]])
    assert scale(1, table=flat) == 3                               # perfect scaling: all the way
    bump = np.array([[10.0, 9.0, 4.0, 8.0]])
    assert scale(1, table=bump) == 1                               # stops at the first count below L, even if a later one recovers


def test_goodput_per_gpu_table():
    wl = W.make("physical")
    c = wl.cfg
    tab = LP.goodput_per_gpu(wl.job_params, wl.m_grid, c.Gs, c.cap, 4)
    for j in (0, 7, 29):
        jb = O.job_from_params(wl.job_params, j)
        assert tab[j, 0] == O.best_goodput(jb, wl.m_grid[j], c.Gs, 1, 1)[0]
        assert tab[j, 1] == O.best_goodput(jb, wl.m_grid[j], c.Gs, c.cap, 1)[0] / c.cap
        assert tab[j, 3] == O.best_goodput(jb, wl.m_grid[j], c.Gs, 3 * c.cap, 3)[0] / (3 * c.cap)
    # a job that pays nothing for synchronisation and whose efficiency does not fall (huge noise scale) scales
    # perfectly as long as the batch-size limits leave room: per-GPU goodput equals the ideal
    jp = wl.job_params.copy()
    jp[2:6] = 0.0
    jp[W.PARAM_INDEX["phi"]] = 1e30
    jp[W.PARAM_INDEX["M0"]] = 1.0
    jp[W.PARAM_INDEX["M_max"]] = 2.0**40
    tab = LP.goodput_per_gpu(jp, wl.m_grid, c.Gs, c.cap, 4)
    assert np.allclose(tab[:, 1:], tab[:, :1], rtol=1e-12)
    assert np.array_equal(LP.autoscale(tab * [1, 1, 1, 1, 1 - 1e-9], np.ones(c.J, np.int32), 2 / 3, 0.5), np.full(c.J, 4))


def test_simulator_tick_bookkeeping():
    wl = W.make("physical")
    c = wl.cfg
    J = c.J
    K = np.array([2] * J, np.int32)
    nodes = np.ones(J, np.int32)
    K[3] = 0                                    # pending job
    K[4], nodes[4] = 6, 2
    changed = np.zeros(J, np.int32)
    changed[5] = 1
    progress = np.full(J, 100.0)
    target = np.full(J, 1e9)
    target[6] = 50.0                            # already finished
    g, new, fin = LP.sim_tick(wl.job_params, wl.m_grid, c.Gs, K, nodes, changed, progress, target, 60.0, 30.0)
    jb = lambda j: O.job_from_params(wl.job_params, j)
    assert g[0] == O.best_goodput(jb(0), wl.m_grid[0], c.Gs, 2, 1)[0] and new[0] == 100.0 + g[0] * 60.0
    assert g[3] == 0.0 and new[3] == 100.0 and not fin[3]
    assert g[4] == O.best_goodput(jb(4), wl.m_grid[4], c.Gs, 6, 2)[0]
    assert new[5] == 100.0 + g[5] * 30.0                            # half of the interval lost to the restart
    assert g[6] == 0.0 and new[6] == 100.0 and fin[6]
    # an interval shorter than the restart delay: a re-allocated job does not move (and never goes backwards)
    _, new2, _ = LP.sim_tick(wl.job_params, wl.m_grid, c.Gs, K, nodes, changed, progress, target, 20.0, 30.0)
    assert new2[5] == 100.0 and new2[0] == 100.0 + g[0] * 20.0
    # reaching the target
    target2 = np.full(J, 100.0 + 0.5 * g[0] * 60.0)
    _, _, fin2 = LP.sim_tick(wl.job_params, wl.m_grid, c.Gs, K, nodes, changed, progress, target2, 60.0, 30.0)
    assert fin2[0]


def test_apply_best_on_a_case_worked_out_by_hand():
    """Three candidates for two jobs on three nodes; fitness ties go to the lower index, NaN ranks last (the
    order of the search step's ranking, checked against it)."""
    pop = np.array([[[1, 0, 0], [0, 2, 0]],
                    [[0, 1, 1], [0, 2, 0]],
                    [[2, 0, 0], [0, 0, 0]]], np.int32)
    cur = np.array([[1, 0, 0], [0, 0, 0]], np.int32)             # job 1 is pending: nothing to restart
    best, new, K, nodes, changed = LP.apply_best(pop, [0.5, 0.9, 0.9], cur)
    assert best == 1 and np.array_equal(new, pop[1])
    assert K.tolist() == [2, 2] and nodes.tolist() == [2, 1] and changed.tolist() == [True, False]
    best, new, K, nodes, changed = LP.apply_best(pop, [np.nan, -3.0, np.nan], cur)
    assert best == 1
    best, new, K, nodes, changed = LP.apply_best(pop, [0.7, 0.1, 0.2], cur)
    assert best == 0 and changed.tolist() == [False, False] and K.tolist() == [1, 2]
    best, *_ = LP.apply_best(pop, [np.nan, np.nan, np.nan], cur)
    assert best == 0
    rng = np.random.default_rng(3)
    for _ in range(50):
        f = rng.choice([0.25, 0.5, np.nan, -2.0, 1.0], 9)
        assert LP.apply_best(np.zeros((9, 1, 1), np.int32), f, np.zeros((1, 1), np.int32))[0] == O.rank(f)[0]
