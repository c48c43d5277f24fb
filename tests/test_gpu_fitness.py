"""GPU parity of pollux_fitness against the CPU oracle (element by element)."""
import numpy as np
import pytest

import workloads as W
from parity import compare, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("name", ["tiny", "physical", "mid"])
def test_fitness_matches_oracle_on_paper_shaped_configs(name):
    wl = W.make(name)
    ties = compare(wl, run_gpu(wl), run_oracle(wl))
    assert ties == 0


@pytest.mark.parametrize("p", [-10.0, -1.0, 0.0, 0.5, 1.0])
def test_fairness_knob_values(p):
    wl = W.make("physical")
    assert compare(wl, run_gpu(wl, p=p), run_oracle(wl, p=p)) == 0


@pytest.mark.parametrize("p", [-1.0, 0.5, 1.0])
def test_mid_config_at_three_knob_values(p):
    wl = W.make("mid")
    sub = wl.population[:200]
    assert compare(wl, run_gpu(wl, population=sub, p=p), run_oracle(wl, population=sub, p=p), population=sub) == 0


def test_fair_share_candidate_scores_exactly_one():
    for name in ("tiny", "physical", "mid"):
        wl = W.make(name, current="fair")
        for p in (-1.0, 0.0, 1.0):
            r = run_gpu(wl, population=wl.population[:1], p=p)
            assert np.all(r["speedup"][0] == 1.0) and r["fitness"][0] == 1.0 and r["status"] == 0


@pytest.mark.parametrize("shape", [
    dict(P=3, J=1, N=1, cap=8, Gm=1, Gs=1),
    dict(P=5, J=7, N=3, cap=4, Gm=5, Gs=3),
    dict(P=9, J=13, N=67, cap=2, Gm=70, Gs=5),        # ragged: N and Gm just past one wavefront
    dict(P=4, J=6, N=130, cap=3, Gm=129, Gs=33),      # grid and s range just past a tile
    dict(P=2, J=3, N=5, cap=4, Gm=200, Gs=70),
    dict(P=1, J=300, N=9, cap=40, Gm=33, Gs=2),       # more jobs than threads of a workgroup
])
def test_ragged_and_degenerate_shapes(shape):
    cfg = W.custom("ragged", **shape)
    wl = W.make(cfg)
    assert compare(wl, run_gpu(wl), run_oracle(wl)) == 0


def test_flags_and_penalty_switch():
    wl = W.make("physical")
    for flags in (1, 2, 3):
        assert compare(wl, run_gpu(wl, flags=flags), run_oracle(wl, flags=flags)) == 0


def test_zero_delta_and_pending_current_jobs():
    wl = W.make("physical")
    cur = wl.current_alloc.copy()
    cur[::3] = 0
    assert compare(wl, run_gpu(wl, current=cur, delta=0.0), run_oracle(wl, current=cur, delta=0.0)) == 0
    assert compare(wl, run_gpu(wl, current=cur), run_oracle(wl, current=cur)) == 0


def test_special_parameter_regimes():
    """gamma = 1 (plain sum), gamma = 10, zeroed synchronisation terms (exploration priors), huge and tiny phi."""
    wl = W.make("physical")
    jp = wl.job_params.copy()
    ix = W.PARAM_INDEX
    jp[ix["gamma"], 0::5] = 1.0
    jp[ix["gamma"], 1::5] = 10.0
    jp[ix["alpha_sync_local"], 2::5] = 0.0
    jp[ix["beta_sync_local"], 2::5] = 0.0
    jp[ix["beta_sync_node"], 3::5] = 0.0
    jp[ix["alpha_sync_node"], 4::10] = 0.0
    jp[ix["beta_sync_node"], 4::10] = 0.0
    jp[ix["phi"], 0::7] = 1e12
    jp[ix["phi"], 3::7] = 1e-3
    assert compare(wl, run_gpu(wl, job_params=jp), run_oracle(wl, job_params=jp), job_params=jp) == 0


def test_tight_batch_limits_and_nothing_feasible():
    wl = W.make("physical")
    jp = wl.job_params.copy()
    ix = W.PARAM_INDEX
    jp[ix["M_max"], 0::4] = jp[ix["M0"], 0::4]            # M must equal M0 exactly
    jp[ix["M0"], 1::8] = 1e7                              # out of reach: goodput 0 everywhere, status ZERO_FAIR
    jp[ix["M_max"], 1::8] = 3.2e8
    jp[ix["M0"], 2::8] = 100.5                            # non-integer limits
    jp[ix["M_max"], 2::8] = 1000.25
    g, r = run_gpu(wl, job_params=jp), run_oracle(wl, job_params=jp)
    assert r["status"] & 2
    assert compare(wl, g, r, job_params=jp) == 0


def test_feasible_windows_that_cut_off_the_unconstrained_optimum_on_either_side():
    """Accumulation counts far beyond one chunk (Gs = 100).  Jobs with a heavy synchronisation cost want many
    accumulation steps but a small M_max allows few; jobs with almost none want s = 0 but a large M0 forbids
    small s: the elected point then sits on the boundary of the feasible window, in whichever chunk that is."""
    cfg = W.custom("windows", P=24, J=30, N=8, cap=8, Gm=70, Gs=100)
    wl = W.make(cfg)
    ix = W.PARAM_INDEX
    jp = wl.job_params.copy()
    jp[ix["alpha_sync_local"], 0::3] = 5.0          # s* large ...
    jp[ix["alpha_sync_node"], 0::3] = 8.0
    jp[ix["M_max"], 0::3] = 4.0 * jp[ix["M0"], 0::3]    # ... but only a few counts are allowed
    jp[ix["alpha_sync_local"], 1::3] = 1e-6         # s* = 0 ...
    jp[ix["beta_sync_local"], 1::3] = 0.0
    jp[ix["alpha_sync_node"], 1::3] = 1e-6
    jp[ix["beta_sync_node"], 1::3] = 0.0
    jp[ix["M0"], 1::3] = 6000.0                     # ... but small batches need many counts
    jp[ix["M_max"], 1::3] = 60000.0
    g, r = run_gpu(wl, job_params=jp), run_oracle(wl, job_params=jp)
    assert compare(wl, g, r, job_params=jp) == 0
    s = r["best_s"]
    assert (s[:, 1::3] >= 8).any() and (s[:, 0::3] >= 1).any() and (s >= 32).any()     # the cases are really there


@pytest.mark.parametrize("P,N,Gm", [(6, 8, 20), (70, 64, 64), (70, 132, 64), (70, 256, 128)])
def test_more_accumulation_counts_than_the_reciprocal_table_kept_on_chip(P, N, Gm):
    """Gs = 300: the table of 1/(s+1) no longer fits the on-chip copy, so the count inside the winning group of
    four and the reciprocal at the clamped count come from memory (with rows of 65 to 256 nodes and whole groups
    of 64 batch sizes the terms of a table row are then read from memory too, not from an on-chip copy; rows of at
    most 64 nodes are then read one to a wavefront load, not four).  Heavy
    synchronisation costs push the elected count far up; M_max is wide enough to allow it."""
    cfg = W.custom("long_s", P=P, J=9, N=N, cap=8, Gm=Gm, Gs=300)
    wl = W.make(cfg)
    ix = W.PARAM_INDEX
    jp = wl.job_params.copy()
    jp[ix["alpha_sync_local"], 0::2] = 10.0
    jp[ix["alpha_sync_node"], 0::2] = 15.0
    jp[ix["phi"], 0::2] = 1e6
    jp[ix["M_max"], :] = 1e7
    g, r = run_gpu(wl, job_params=jp), run_oracle(wl, job_params=jp)
    assert compare(wl, g, r, job_params=jp) == 0
    s = r["best_s"]
    assert ((s >= 100) & (s < 256)).any() and (s < 32).any()     # inside the range, not only at its end
    assert Gm > 64 or ((s >= 256) & (s < 299)).any()              # (the grid of 128 batch sizes elects none that far up)


def test_status_bits():
    wl = W.make("tiny")
    ix = W.PARAM_INDEX
    jp = wl.job_params.copy()
    jp[ix["gamma"], 2] = 11.0
    assert run_gpu(wl, job_params=jp)["status"] & 1
    jp = wl.job_params.copy()
    jp[ix["age_T"], 1] = 10.0
    jp[ix["restarts_R"], 1] = 3.0
    g, r = run_gpu(wl, job_params=jp), run_oracle(wl, job_params=jp)
    assert g["status"] == r["status"] == 4
    pop = wl.population.copy()
    pop[2, 2, 1] = -1
    assert run_gpu(wl, population=pop)["status"] == 8


@pytest.mark.parametrize("flags", [0, 4])
@pytest.mark.parametrize("shape", [dict(P=37, J=11, N=64, cap=8, Gm=64, Gs=16), dict(P=21, J=9, N=16, cap=4, Gm=64, Gs=8),
                                   dict(P=522, J=200, N=64, cap=8, Gm=64, Gs=16)])       # the last: several candidates per wavefront
def test_negative_entries_in_rows_of_at_most_64_nodes(shape, flags):
    """Rows of at most 64 nodes are read four to a wavefront load.  A negative entry (invalid input) is
    flagged, and K, the node count, the penalty and the per-node totals still follow the plain definitions
    (the entry counts as it is), as in the oracle; plain and memoised (flags = 4)."""
    cfg = W.custom("neg64", **shape)
    wl = W.make(cfg)
    pop = wl.population.copy()
    rng = np.random.default_rng(5)
    for cand in (0, 3, 4, 5, 6, cfg.P - 1):
        for j in rng.choice(cfg.J, size=3, replace=False):
            n = int(rng.integers(cfg.N))
            pop[cand, j, n] = -int(rng.integers(1, 3))
            pop[cand, j, (n + 5) % cfg.N] += 3          # most of these rows keep K >= 1
    g, r = run_gpu(wl, population=pop, flags=flags), run_oracle(wl, population=pop)
    assert g["status"] & 8 and r["status"] & 8
    assert compare(wl, g, r, population=pop) == 0


@pytest.mark.parametrize("flags", [0, 4])
def test_out_of_range_entries_in_rows_of_65_to_256_nodes(flags):
    """Rows of 65 to 256 nodes are read one to a wavefront load, and the sums of two rows come out of one
    reduction while every entry lies in 0 .. 255.  Negative entries and entries far beyond that range (invalid
    input, flagged or counted as violations) take the other path: planted in the first and in the second row of
    a pair, in both rows, in the first and in the last eight candidates of a wavefront and in the ragged tail
    of the population; K, the node count and the per-node totals follow the plain definitions, as in the oracle."""
    cfg = W.custom("wide132", P=2003, J=200, N=132, cap=8, Gm=64, Gs=8)
    wl = W.make(cfg)
    pop = wl.population.copy()
    rng = np.random.default_rng(11)
    # the candidates of one wavefront are 4 apart: 0, 4, 8, ... are its candidates 0, 1, 2, ...
    for cand, value in ((0, -2), (12, 300), (16, 70000), (20, -1), (36, 256), (40, -3), (44, 1000), (60, -1),
                        (61, 255), (65, -2), (cfg.P - 1, 400), (cfg.P - 2, -1)):
        for j in rng.choice(cfg.J, size=5, replace=False):
            n = int(rng.integers(cfg.N))
            pop[cand, j, n] = value
            pop[cand, j, (n + 7) % cfg.N] += 2
    g, r = run_gpu(wl, population=pop, flags=flags), run_oracle(wl, population=pop)
    assert g["status"] & 8 and r["status"] & 8
    assert compare(wl, g, r, population=pop) == 0


def test_a_job_without_gradient_time_is_flagged_and_leaves_the_other_jobs_alone():
    """alpha_grad = beta_grad = 0 (T_grad = 0, outside the model's domain): status bit on both sides, the
    call completes, and every other job's elected point and goodput still match the oracle."""
    wl = W.make("physical")
    ix = W.PARAM_INDEX
    jp = wl.job_params.copy()
    bad = 5
    jp[ix["alpha_grad"], bad] = 0.0
    jp[ix["beta_grad"], bad] = 0.0
    g, r = run_gpu(wl, job_params=jp), run_oracle(wl, job_params=jp)
    assert g["status"] & 1 and r["status"] & 1
    others = np.arange(wl.cfg.J) != bad
    for k in ("best_m", "best_s"):
        assert np.array_equal(g[k][:, others], r[k][:, others])
    for k in ("best_goodput", "speedup"):
        assert np.allclose(g[k][:, others], r[k][:, others], rtol=1e-12, atol=0.0)


def test_starved_jobs_and_duplicate_batch_sizes():
    wl = W.make("tiny")
    pop = wl.population.copy()
    pop[:, 5, :] = 0
    for p in (-1.0, 0.0, 1.0):
        assert compare(wl, run_gpu(wl, population=pop, p=p), run_oracle(wl, population=pop, p=p), population=pop) == 0
    # a grid made of copies of few values: ties must go to the lowest index on both sides
    wl.m_grid[:] = np.repeat(wl.m_grid[:, ::8], 8, axis=1)
    assert compare(wl, run_gpu(wl), run_oracle(wl)) == 0


@pytest.mark.parametrize("Gm", [64, 128])
def test_duplicate_batch_sizes_in_grids_of_one_and_two_groups_of_64(Gm):
    """Rows of 65 to 256 nodes with a grid of 64 or 128 batch sizes: the sweep takes the grid in one or two groups
    of 64, one batch size per lane.  Grids made of copies put equal goodput values into several lanes of a group,
    into the same lane of both groups, and into both (whichever copy wins, m* and s* are the same values); a grid
    with its halves exchanged, or reversed, moves the best points into the other group and to the other end of the
    lanes.  Elected (m*, s*), goodput and fitness must match the oracle in every case."""
    cfg = W.custom("wide_ties", P=301, J=48, N=132, cap=8, Gm=Gm, Gs=32)
    wl = W.make(cfg)
    base = wl.m_grid.copy()
    grids = [np.concatenate([base[:, :64]] * (Gm // 64), axis=1),                    # the second group repeats the first
             np.repeat(base[:, ::4], 4, axis=1),                                      # runs of four equal batch sizes
             np.concatenate([base[:, :32]] * (Gm // 32), axis=1),                     # lanes l and l + 32, and both groups
             np.concatenate([base[:, 64:], base[:, :64]], axis=1) if Gm == 128 else base[:, ::-1].copy()]   # best point late in the grid
    for grid in grids:
        wl.m_grid[:] = grid
        assert compare(wl, run_gpu(wl), run_oracle(wl)) == 0


def test_deterministic_across_runs():
    wl = W.make("physical")
    a, b = run_gpu(wl), run_gpu(wl)
    for k in ("fitness", "best_m", "best_s", "best_goodput", "speedup", "violations"):
        assert np.array_equal(a[k], b[k], equal_nan=True)


def test_large_config_on_sampled_candidates():
    """Headline shape (1000 jobs, 256 nodes, 128 x 32 grid) on a seeded subset of its population."""
    cfg = W.CONFIGS["large"]
    wl = W.make(cfg, with_population=False)
    rng = np.random.default_rng(64)
    spoiled = [i for i in range(cfg.P) if i % 20 == 7]              # overloaded nodes, several multi-node jobs per node
    pending = [i for i in range(cfg.P) if i % 10 == 3]              # jobs without GPUs
    idx = sorted(set([0, 1, 1000, 4095] + list(rng.choice(spoiled, 12, replace=False)) +
                     list(rng.choice(pending, 12, replace=False)) + list(rng.integers(0, cfg.P, 44))))
    assert len(idx) >= 64
    sub = np.concatenate([W.candidates(cfg, int(i), 1) for i in idx])
    ref = run_oracle(wl, population=sub)
    assert (ref["violations"] > 0).sum() >= 12 and ((sub.sum(2) == 0).any(1)).sum() >= 12
    assert compare(wl, run_gpu(wl, population=sub), ref, population=sub) == 0


@pytest.mark.parametrize("p", [-1.0, 0.5, 1.0])
def test_fp32_variant_on_the_mid_configuration(p):
    """precision = 1: fp32 arithmetic checked against the fp64 oracle.  Goodput, SPEEDUP and fitness within
    1e-5 relative; the GPU's (m, s) may differ from the oracle's where fp32 cannot separate two points, but
    the oracle's goodput at the GPU's choice must be within 1e-5 of the oracle's maximum."""
    import oracle as O
    wl = W.make("mid")
    sub = wl.population[:300]
    g = run_gpu(wl, population=sub, p=p, precision=1)
    r = run_oracle(wl, population=sub, p=p)
    assert g["status"] == r["status"] and np.array_equal(g["violations"], r["violations"])
    from parity import rel_err
    for name in ("best_goodput", "speedup", "fitness"):
        assert rel_err(g[name], r[name]).max() <= 1e-5, name
    differ = np.argwhere((g["best_m"] != r["best_m"]) | (g["best_s"] != r["best_s"]))
    agreement = 1.0 - len(differ) / g["best_m"].size
    print(f"fp32 (m,s) agreement with the fp64 oracle at p={p}: {agreement:.6f} ({len(differ)} of {g['best_m'].size} differ)")
    assert agreement > 0.99
    for cand, j in differ[:500]:
        K, nodes = int(sub[cand, j].sum()), int((sub[cand, j] > 0).sum())
        at, ok = O.goodput(O.job_from_params(wl.job_params, j), K, nodes, int(g["best_m"][cand, j]), int(g["best_s"][cand, j]))
        assert ok and abs(at - r["best_goodput"][cand, j]) <= 1e-5 * r["best_goodput"][cand, j]


def test_fp32_variant_small_and_ragged():
    from parity import rel_err
    for cfg in (W.CONFIGS["tiny"], W.custom("ragged32", P=4, J=6, N=130, cap=3, Gm=129, Gs=33)):
        wl = W.make(cfg)
        g, r = run_gpu(wl, precision=1), run_oracle(wl)
        assert np.array_equal(g["violations"], r["violations"])
        for name in ("best_goodput", "speedup", "fitness"):
            assert rel_err(g[name], r[name]).max() <= 1e-5, name
    wl = W.make("tiny", current="fair")
    g = run_gpu(wl, population=wl.population[:1], precision=1)
    assert g["fitness"][0] == 1.0 and np.all(g["speedup"][0] == 1.0)


def test_large_config_full_population_in_the_benchmark_launch_shape():
    """All 4096 candidates on the GPU (the launch configuration bench.py times: 64 000 workgroups, 16 candidates
    per wavefront) against the oracle on all 4096 (4.1 million pairs, each a sweep of 4096 grid points)."""
    import torch
    import paper_2008_12260_amd as px
    cfg = W.CONFIGS["large"]
    wl = W.make(cfg, with_population=False)
    pop = W.candidates(cfg, 0, cfg.P)
    call = px.FitnessCall(cfg.P, cfg.J, cfg.N, cfg.Gm, cfg.Gs, wl.job_params, wl.m_grid, wl.fair_share,
                          wl.current_alloc, wl.node_capacity, p=cfg.p, delta=cfg.delta)
    dpop = torch.from_numpy(pop).cuda()
    call.run(dpop, outputs="fitness")           # as a search loop calls it: nothing per pair written
    lean = {k: v.copy() for k, v in call.results().items() if k in ("fitness", "violations")}
    call.run(dpop, outputs="argmax")            # as bench.py's headline loop calls it: no per-pair goodput or speedup
    lean.update({k: v.copy() for k, v in call.results().items() if k in ("best_m", "best_s")})
    for k in ("fitness", "violations"):
        assert np.array_equal(lean[k], call.results()[k], equal_nan=True), k
    call.run(dpop)
    g = call.results()
    for k, v in lean.items():
        assert np.array_equal(v, g[k], equal_nan=True), k
    r = run_oracle(wl, population=pop)
    assert compare(wl, g, r, population=pop) == 0
    # properties that hold at any size: infeasible candidates are exactly the spoiled slice and score -V;
    # every feasible candidate has a finite fitness >= 0; the argmax respects the batch-size limits
    bad = np.flatnonzero(g["violations"] > 0)
    assert set(bad) <= {i for i in range(cfg.P) if i % 20 == 7}
    assert np.array_equal(g["fitness"][bad], -g["violations"][bad].astype(np.float64))
    good = g["violations"] == 0
    assert np.all(np.isfinite(g["fitness"][good])) and np.all(g["fitness"][good] >= 0)
    K = pop.sum(2)
    have = g["best_m"] > 0
    M = K * g["best_m"] * (g["best_s"] + 1)
    assert np.all(M[have] >= wl.param("M0")[None].repeat(cfg.P, 0)[have])
    assert np.all(M[have] <= wl.param("M_max")[None].repeat(cfg.P, 0)[have])
    assert np.all((g["best_goodput"] > 0) == have)


@pytest.mark.parametrize("name", ["tiny", "physical", "mid"])
def test_memoised_mode_gives_the_same_results(name):
    """PX_FLAG_MEMOISE: one sweep per (job, K, placement class), looked up per pair."""
    wl = W.make(name)
    g = run_gpu(wl, flags=4)
    assert compare(wl, g, run_oracle(wl)) == 0
    plain = run_gpu(wl)
    for k in ("fitness", "best_m", "best_s", "best_goodput", "speedup", "violations"):
        assert np.array_equal(g[k], plain[k], equal_nan=True), k


@pytest.mark.parametrize("shape", [dict(P=7, J=70, N=128, cap=2, Gm=20, Gs=6),          # a second, partly filled tile of jobs
                                   dict(P=5, J=21, N=68, cap=40, Gm=33, Gs=5),          # K beyond the memo table
                                   dict(P=3, J=130, N=256, cap=8, Gm=64, Gs=32),
                                   dict(P=3, J=1100, N=68, cap=40, Gm=8, Gs=4),          # more jobs than one finishing step takes
                                   dict(P=2, J=2051, N=72, cap=30, Gm=5, Gs=3)])
def test_memoised_mode_on_rows_of_65_to_256_nodes(shape):
    """These rows take the memoised pass that walks the population candidate by candidate; negative entries in a
    few rows as well (flagged, counted as they are)."""
    cfg = W.custom("memo_rows", **shape)
    wl = W.make(cfg)
    g = run_gpu(wl, flags=4)
    assert compare(wl, g, run_oracle(wl)) == 0
    plain = run_gpu(wl)
    for k in ("fitness", "best_m", "best_s", "best_goodput", "speedup", "violations"):
        assert np.array_equal(g[k], plain[k], equal_nan=True), k
    pop = wl.population.copy()
    pop[0, 1, 3] = -1
    pop[cfg.P - 1, cfg.J - 1, cfg.N - 1] = -2
    pop[cfg.P - 1, cfg.J - 1, 0] += 4
    pop[cfg.P - 1, cfg.J - 2, 2] += 70                    # and two rows with more GPUs than the memo table covers
    pop[1, cfg.J // 2, cfg.N - 2] += 90
    g, r = run_gpu(wl, population=pop, flags=4), run_oracle(wl, population=pop)
    assert g["status"] & 8 and r["status"] & 8
    assert compare(wl, g, r, population=pop) == 0


@pytest.mark.parametrize("N", [68, 128, 256])
def test_memoised_mode_tells_changed_rows_from_unchanged_ones(N):
    """The re-allocation penalty hinges on whether a row equals the job's current row.  Candidates built from the
    current allocation itself: unchanged; the same nodes with other counts; a GPU moved to the neighbouring node
    (same 16-byte group of the row, or the next group); moved to the far end of the row; a job that holds
    nothing now and gets GPUs; a job that holds GPUs now and gets none.  Plain and memoised mode, against the
    oracle's SPEEDUP (the factor is far from 1 for these jobs)."""
    cfg = W.custom("changed_rows", P=8, J=70, N=N, cap=8, Gm=20, Gs=6)
    wl = W.make(cfg)
    cur = wl.current_alloc.copy()
    cur[5] = 0                                              # job 5 holds nothing now
    jp = wl.job_params.copy()
    jp[11] = 600.0                                          # T_j: young jobs, so that the penalty is large
    jp[12] = 3.0                                            # R_j
    pop = np.repeat(cur[None], cfg.P, 0).copy()
    rng = np.random.default_rng(5)
    changed = np.zeros((cfg.P, cfg.J), bool)
    for j in range(cfg.J):
        occ = np.flatnonzero(cur[j])
        if len(occ) == 0:
            continue
        n = int(occ[0])
        pop[1, j, n] += 1                                   # same nodes, another count
        to = n + 1 if n + 1 < N and cur[j, n + 1] == 0 else n
        pop[2, j, n] -= 1; pop[2, j, to] += 1               # one GPU to the next node
        far = N - 1 - n if cur[j, N - 1 - n] == 0 else n
        pop[3, j, n] -= 1; pop[3, j, far] += 1              # one GPU to the mirrored node
        pop[4, j] = 0                                       # gets nothing
        pop[6, j] = np.roll(cur[j], 4)                      # every entry one 16-byte group further
        if rng.uniform() < 0.5:
            pop[7, j] = np.roll(cur[j], 1)
    pop[5, 5, 3] = 2                                        # the job that holds nothing now gets GPUs
    changed = (pop != cur[None]).any(2)
    assert changed[1:5].mean() > 0.9 and not changed[0].any()
    r = run_oracle(wl, population=pop, current=cur, job_params=jp, flags=2)
    for flags in (2, 2 | 4):                                # constraint check off: the matrices overload nodes
        g = run_gpu(wl, population=pop, current=cur, job_params=jp, flags=flags)
        assert compare(wl, g, r, population=pop, job_params=jp) == 0
    # and the penalty is what tells the rows apart: unchanged rows score the plain ratio
    plain = run_oracle(wl, population=pop, current=pop[0], job_params=jp, flags=2 | 1)
    live = cur.sum(1) > 0
    assert np.array_equal(r["speedup"][0], plain["speedup"][0])
    assert np.all(r["speedup"][1][live] < plain["speedup"][1][live])


def test_memoised_mode_with_rows_beyond_the_table_and_in_fp32():
    cfg = W.custom("bigK", P=6, J=40, N=9, cap=40, Gm=33, Gs=5)      # K up to 160: beyond the 64-entry table
    wl = W.make(cfg)
    assert wl.population.sum(2).max() > 64
    assert compare(wl, run_gpu(wl, flags=4), run_oracle(wl)) == 0
    wl = W.make("physical")
    a, b = run_gpu(wl, flags=4, precision=1), run_gpu(wl, precision=1)
    for k in ("fitness", "best_m", "best_s", "best_goodput", "speedup"):
        assert np.array_equal(a[k], b[k], equal_nan=True), k


@pytest.mark.parametrize("name", ["physical", "mid"])
def test_rows_that_claim_more_gpus_on_one_node_than_any_node_has(name):
    """The tables of the one-node class stop at the largest node capacity; a row beyond it (which no valid
    allocation has) is swept in place.  Plain, memoised, sampling and fp32 calls on a population with many such
    rows, next to ordinary ones, at every count up to the tables' end and beyond."""
    from parity import rel_err
    wl = W.make(name)
    c = wl.cfg
    pop = wl.population[:48].copy()
    cap = int(wl.node_capacity.max())
    rng = np.random.default_rng(7)
    for cand in range(0, pop.shape[0], 2):
        for j in rng.choice(c.J, size=c.J // 3, replace=False):
            pop[cand, j] = 0
            pop[cand, j, rng.integers(c.N)] = rng.integers(cap + 1, 70)          # one node, up to beyond kTableK
    ref = run_oracle(wl, population=pop)
    assert ref["violations"].max() > 0
    assert compare(wl, run_gpu(wl, population=pop), ref, population=pop) == 0
    assert compare(wl, run_gpu(wl, population=pop, flags=4), ref, population=pop) == 0
    sw = W.sampled(wl)
    sref = run_oracle(sw, population=pop, flags=16)
    assert compare(sw, run_gpu(sw, population=pop, flags=16), sref, population=pop, sampled=True) == 0
    assert compare(sw, run_gpu(sw, population=pop, flags=16 | 4), sref, population=pop, sampled=True) == 0
    g = run_gpu(wl, population=pop, precision=1)
    for k in ("best_goodput", "speedup"):
        assert rel_err(g[k], ref[k]).max() <= 1e-5, k
    gm = run_gpu(wl, population=pop, precision=1, flags=4)
    for k in ("fitness", "best_m", "best_s", "best_goodput", "speedup"):
        assert np.array_equal(g[k], gm[k], equal_nan=True), k


def test_keep_job_tables_reuses_the_job_level_work():
    """PX_FLAG_KEEP_JOB_TABLES: a second call on the same workspace with another population skips the job-level
    kernels and must give what a full call gives."""
    import torch
    import paper_2008_12260_amd as px
    for flags in (0, px.PX_FLAG_MEMOISE):
        wl = W.make("mid")
        c = wl.cfg
        call = px.FitnessCall(c.P, c.J, c.N, c.Gm, c.Gs, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc,
                              wl.node_capacity, p=c.p, delta=c.delta, flags=flags)
        first = torch.as_tensor(wl.population).cuda()
        other = torch.as_tensor(np.ascontiguousarray(wl.population[::-1])).cuda()
        crowded = torch.as_tensor(np.ascontiguousarray(wl.population * 3)).cuda()      # over capacity on many nodes
        call.run(first)
        call.run(crowded, keep_job_tables=True)       # leaves no trace in the per-node counters of the next call
        assert call.results()["violations"].max() > 0
        call.run(other, keep_job_tables=True)
        kept = call.results()
        call.run(other)
        full = call.results()
        for k in ("fitness", "best_m", "best_s", "best_goodput", "speedup", "violations", "status"):
            assert np.array_equal(kept[k], full[k], equal_nan=True), k


# ---- the sampling argmax of Sec. 4.3 (PX_FLAG_SAMPLE_M) -------------------------------------------------------

@pytest.mark.parametrize("name", ["tiny", "physical", "mid"])
def test_sampling_argmax_matches_oracle(name):
    wl = W.sampled(W.make(name))
    pop = wl.population[:300]
    ref = run_oracle(wl, population=pop, flags=16)
    assert (ref["best_m"] > 0).mean() > 0.5                      # the workload exercises the procedure
    assert compare(wl, run_gpu(wl, population=pop, flags=16), ref, population=pop, sampled=True) == 0


@pytest.mark.parametrize("shape", [
    dict(P=3, J=1, N=1, cap=8, Gm=1, Gs=1),
    dict(P=9, J=13, N=67, cap=2, Gm=70, Gs=5),
    dict(P=4, J=6, N=130, cap=3, Gm=129, Gs=33),
    dict(P=6, J=40, N=9, cap=40, Gm=33, Gs=5),                   # K beyond the memo table
])
def test_sampling_argmax_on_ragged_shapes_plain_and_memoised(shape):
    wl = W.sampled(W.make(W.custom("ragged_sampled", **shape)))
    ref = run_oracle(wl, flags=16)
    plain = run_gpu(wl, flags=16)
    assert compare(wl, plain, ref, sampled=True) == 0
    memo = run_gpu(wl, flags=16 | 4)
    for k in ("fitness", "best_m", "best_s", "best_goodput", "speedup", "violations", "status"):
        assert np.array_equal(memo[k], plain[k], equal_nan=True), k


def test_sampling_argmax_flags_a_bad_memory_bound_and_rejects_fp32():
    import paper_2008_12260_amd as px
    wl = W.sampled(W.make("tiny"))
    jp = wl.job_params.copy()
    jp[W.PARAM_INDEX["m_mem"], 2] = 0.0
    g, ref = run_gpu(wl, flags=16, job_params=jp), run_oracle(wl, flags=16, job_params=jp)
    assert g["status"] == ref["status"] and g["status"] & 1
    with pytest.raises(px.PolluxError):
        run_gpu(wl, flags=16, precision=1)


def test_non_adaptive_jobs_with_a_fixed_batch_size():
    """M_max = M0 for every job (Sec. 4.1, jobs that do not adapt their batch size): only exact splits of M0 are
    feasible and EFFICIENCY is 1; the grid lists the divisors."""
    cfg = W.custom("fixed_batch", P=64, J=24, N=8, cap=4, Gm=16, Gs=8)
    wl = W.make(cfg)
    jp = wl.job_params.copy()
    jp[W.PARAM_INDEX["M_max"]] = jp[W.PARAM_INDEX["M0"]]
    wl.m_grid[:] = np.array([1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64, 96, 128, 192, 256], np.int32)
    ref = run_oracle(wl, job_params=jp)
    g = run_gpu(wl, job_params=jp)
    assert compare(wl, g, ref, job_params=jp) == 0
    have = g["best_m"] > 0
    assert have.mean() > 0.3
    K = wl.population.sum(2)
    assert np.all((K * g["best_m"] * (g["best_s"] + 1))[have] == np.broadcast_to(jp[W.PARAM_INDEX["M0"]], K.shape)[have])


# ---- launch-shape corners of the pairs kernel -----------------------------------------------------------------

@pytest.mark.parametrize("shape", [
    dict(P=5, J=7, N=260, cap=2, Gm=20, Gs=6),        # rows of 16-byte groups beyond one wavefront's single load
    dict(P=3, J=4, N=512, cap=1, Gm=9, Gs=3),
    dict(P=6, J=5, N=256, cap=2, Gm=64, Gs=32),       # exactly one load per lane, one full mask group
    dict(P=6, J=5, N=252, cap=2, Gm=65, Gs=31),       # one lane short of it, grid one past it
])
def test_row_lengths_around_the_single_load_case(shape):
    wl = W.make(W.custom("rows", **shape))
    assert compare(wl, run_gpu(wl), run_oracle(wl)) == 0


def test_several_candidates_per_wavefront_with_a_ragged_population():
    """P * J large enough for several candidates per wavefront, P not a multiple of a workgroup's share."""
    cfg = W.custom("ragged_population", P=1001, J=200, N=64, cap=8, Gm=64, Gs=16)
    wl = W.make(cfg)
    ref = run_oracle(wl)
    for flags in (0, 4):
        assert compare(wl, run_gpu(wl, flags=flags), ref) == 0


def test_population_that_is_not_16_byte_aligned():
    """A population view that starts 4 bytes into its allocation takes the scalar row path."""
    import torch
    import paper_2008_12260_amd as px
    wl = W.make("physical")
    c = wl.cfg
    call = px.FitnessCall(c.P, c.J, c.N, c.Gm, c.Gs, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc,
                          wl.node_capacity, p=c.p, delta=c.delta)
    flat = torch.zeros(wl.population.size + 1, dtype=torch.int32, device="cuda")
    view = flat[1:].view(c.P, c.J, c.N)
    view.copy_(torch.as_tensor(wl.population))
    assert view.data_ptr() % 16 == 4
    call.run(view)
    assert compare(wl, call.results(), run_oracle(wl)) == 0


def test_many_random_shapes_and_parameter_draws():
    """Forty seeded configurations with shapes and seeds of their own (grid sizes around the wavefront and chunk
    boundaries, duplicate-heavy grids, few and many GPUs per node).  The election of (m*, s*) must agree with
    the oracle everywhere; a disagreement is tolerated only as a tie below fp64 resolution, which compare()
    verifies against the oracle in extended precision and counts."""
    rng = np.random.default_rng(2024)
    ties = 0
    for trial in range(40):
        shape = dict(P=int(rng.integers(1, 12)), J=int(rng.integers(1, 40)), N=int(rng.choice([1, 2, 3, 4, 8, 16, 63, 64, 65, 256])),
                     cap=int(rng.choice([1, 2, 4, 8, 16])), Gm=int(rng.choice([1, 2, 7, 31, 63, 64, 65, 127, 128, 129, 200])),
                     Gs=int(rng.choice([1, 2, 3, 7, 8, 9, 15, 16, 17, 31, 32, 33, 64, 65])), index=200 + trial)
        wl = W.make(W.custom(f"random{trial}", **shape))
        p = float(rng.choice([-2.0, -1.0, 0.0, 1.0]))
        ref = run_oracle(wl, p=p)
        for flags in (0, 4):
            ties += compare(wl, run_gpu(wl, p=p, flags=flags), ref)
    assert ties == 0


def test_random_mid_sized_shapes_with_several_candidates_per_wavefront():
    """Sixteen seeded configurations large enough that a wavefront walks several candidates (ragged counts of
    candidates, rows of 4 to 256 nodes, grids around the wavefront and chunk sizes), a third of them with a few
    negative entries; plain and memoised, bit-exact elections."""
    rng = np.random.default_rng(11)
    ties = 0
    for trial in range(16):
        shape = dict(P=int(rng.integers(150, 1400)), J=int(rng.integers(40, 220)),
                     N=int(rng.choice([4, 8, 16, 32, 60, 64, 68, 128, 256])), cap=int(rng.choice([2, 4, 8])),
                     Gm=int(rng.choice([31, 63, 64, 65, 128])), Gs=int(rng.choice([7, 8, 16, 17, 32, 33])), index=900 + trial)
        wl = W.make(W.custom(f"several{trial}", **shape))
        p = float(rng.choice([-1.0, 0.0, 1.0]))
        pop = wl.population
        if trial % 3 == 0:
            pop = pop.copy()
            for _ in range(20):
                pop[rng.integers(shape["P"]), rng.integers(shape["J"]), rng.integers(shape["N"])] -= 2
        ref = run_oracle(wl, population=pop, p=p)
        for flags in (0, 4):
            ties += compare(wl, run_gpu(wl, population=pop, p=p, flags=flags), ref, population=pop)
    assert ties == 0
