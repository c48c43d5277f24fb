"""GPU parity of the auto-scaling calls (Sec. 5.3.3) and of the simulator tick (Sec. 5.3) with the CPU checker."""
import numpy as np
import pytest

import oracle.loop as LP
import workloads as W
from parity import rel_err

pytestmark = pytest.mark.gpu
RTOL = 1e-12


def device_call(wl):
    import paper_2008_12260_amd as px
    c = wl.cfg
    return px.FitnessCall(1, c.J, 1, c.Gm, c.Gs, wl.job_params, wl.m_grid, wl.fair_share, np.zeros((c.J, 1), np.int32),
                          np.ones(1, np.int32), p=c.p, delta=c.delta)


@pytest.mark.parametrize("name,max_nodes", [("tiny", 4), ("physical", 16), ("mid", 12)])
def test_goodput_per_gpu_and_autoscale(name, max_nodes):
    import torch
    import paper_2008_12260_amd as px
    wl = W.make(name, with_population=False)
    c = wl.cfg
    call = device_call(wl)
    per_gpu = torch.empty((c.J, max_nodes + 1), dtype=torch.float64, device="cuda")
    px.pollux_goodput_per_gpu(call.dims, call.job_params, call.m_grid, c.cap, max_nodes, call.workspace, per_gpu)
    want = LP.goodput_per_gpu(wl.job_params, wl.m_grid, c.Gs, c.cap, max_nodes)       # K up to 16 x 8 = 128: beyond the tables
    got = per_gpu.cpu().numpy()
    assert rel_err(got, want).max() <= RTOL
    rng = np.random.default_rng(31)
    now = rng.integers(0, max_nodes + 2, c.J).astype(np.int32)
    for U, L in ((2 / 3, 0.5), (0.5, 0.25), (0.9, 0.8)):
        new = torch.empty(c.J, dtype=torch.int32, device="cuda")
        px.pollux_autoscale(per_gpu, torch.as_tensor(now).cuda(), U, L, new)
        # the decision is taken on the library's own table (bit-exact rule); on the checker's table it may differ
        # only where a comparison is decided by the last places of two goodput values
        assert np.array_equal(new.cpu().numpy(), LP.autoscale(got, now, U, L))
        other = LP.autoscale(want, now, U, L)
        differ = np.flatnonzero(new.cpu().numpy() != other)
        for j in differ:
            margins = np.concatenate([np.abs(want[j, 1:] / want[j, 0] - U), np.abs(want[j, 1:] / want[j, 0] - L)])
            assert margins.min() < 1e-9, j
        assert len(differ) <= 1


def test_autoscale_grows_a_job_as_its_noise_scale_grows():
    """The behaviour the paper reports: later in training (larger gradient noise scale) more nodes pay off."""
    import torch
    import paper_2008_12260_amd as px
    wl = W.make("physical", with_population=False)
    c = wl.cfg
    sizes = []
    for phi in (1e2, 1e4, 1e6):
        jp = wl.job_params.copy()
        jp[W.PARAM_INDEX["phi"]] = phi
        import dataclasses
        call = device_call(dataclasses.replace(wl, job_params=jp))
        per_gpu = torch.empty((c.J, 17), dtype=torch.float64, device="cuda")
        px.pollux_goodput_per_gpu(call.dims, call.job_params, call.m_grid, c.cap, 16, call.workspace, per_gpu)
        new = torch.empty(c.J, dtype=torch.int32, device="cuda")
        px.pollux_autoscale(per_gpu, torch.ones(c.J, dtype=torch.int32, device="cuda"), 2 / 3, 0.5, new)
        sizes.append(new.cpu().numpy())
    assert np.all(sizes[0] <= sizes[1]) and np.all(sizes[1] <= sizes[2]) and sizes[2].sum() > sizes[0].sum()


@pytest.mark.parametrize("name", ["physical", "mid"])
def test_simulator_tick(name):
    import torch
    import paper_2008_12260_amd as px
    wl = W.make(name)
    c = wl.cfg
    call = device_call(wl)
    rng = np.random.default_rng(32)
    alloc = wl.population[5]                                   # some candidate's allocation
    K = alloc.sum(1).astype(np.int32)
    nodes = (alloc > 0).sum(1).astype(np.int32)
    K[::11] = 0
    changed = (rng.uniform(size=c.J) < 0.3).astype(np.int32)
    progress = rng.uniform(0, 1e6, c.J)
    target = progress + rng.uniform(-1e4, 5e5, c.J)            # some already finished, some finishing now
    dev = lambda a: torch.as_tensor(a).cuda()
    d_progress = dev(progress)
    goodput = torch.empty(c.J, dtype=torch.float64, device="cuda")
    finished = torch.empty(c.J, dtype=torch.int32, device="cuda")
    state = progress
    for dt in (60.0, 60.0, 10.0):                              # three intervals, the last shorter than the restart delay
        px.pollux_sim_tick(call.dims, call.job_params, call.m_grid, dev(K), dev(nodes), dev(changed), dev(target), dt, 30.0,
                           call.workspace, d_progress, goodput, finished)
        g, new, fin = LP.sim_tick(wl.job_params, wl.m_grid, c.Gs, K, nodes, changed, state, target, dt, 30.0)
        assert rel_err(goodput.cpu().numpy(), g).max() <= RTOL
        got = d_progress.cpu().numpy()
        assert rel_err(got, new).max() <= RTOL
        near = np.abs(new - target) <= 1e-9 * np.abs(target)   # the finish line decided by the last places
        assert np.array_equal(finished.cpu().numpy().astype(bool)[~near], fin[~near])
        assert np.all(got >= state)
        state = got                                            # the next interval starts from the library's state


def test_argument_checks():
    import torch
    import paper_2008_12260_amd as px
    wl = W.make("tiny", with_population=False)
    c = wl.cfg
    call = device_call(wl)
    out = torch.empty((c.J, 5), dtype=torch.float64, device="cuda")
    with pytest.raises(px.PolluxError):
        px.pollux_goodput_per_gpu(call.dims, call.job_params, call.m_grid, 0, 4, call.workspace, out)
    with pytest.raises(px.PolluxError):
        px.pollux_goodput_per_gpu(call.dims, call.job_params, call.m_grid, 4, 0, call.workspace, out)
    bad = px.Dims(1, c.J, 1, c.Gm, c.Gs, 1, 0)                 # fp32 is not offered here
    with pytest.raises(px.PolluxError):
        px.pollux_goodput_per_gpu(bad, call.job_params, call.m_grid, 4, 4, call.workspace, out)
    z = torch.zeros(c.J, dtype=torch.int32, device="cuda")
    with pytest.raises(px.PolluxError):
        px.pollux_autoscale(out, z, float("nan"), 0.5, z.clone())


@pytest.mark.parametrize("name", ["tiny", "physical", "mid"])
def test_apply_best_matches_the_checker(name):
    import torch
    import paper_2008_12260_amd as px
    wl = W.make(name)
    c = wl.cfg
    rng = np.random.default_rng(41)
    dev = lambda a: torch.as_tensor(np.ascontiguousarray(a)).cuda()
    pop = dev(wl.population)
    for case in range(4):
        fit = rng.choice([0.3, 0.8, 0.8, -2.0, np.nan], c.P) if case < 2 else rng.uniform(size=c.P)
        if case == 3:
            fit[:] = np.nan
        cur = wl.current_alloc.copy()
        cur[::3] = 0                                            # pending jobs: nothing to restart
        d_cur = dev(cur)
        best = torch.empty(1, dtype=torch.int32, device="cuda")
        K, nodes, changed = (torch.empty(c.J, dtype=torch.int32, device="cuda") for _ in range(3))
        px.pollux_apply_best(px.Dims(c.P, c.J, c.N, 0, 0, 0, 0), pop, dev(fit), d_cur, best, K, nodes, changed)
        w_best, w_new, w_K, w_nodes, w_changed = LP.apply_best(wl.population, fit, cur)
        assert int(best.item()) == w_best
        assert np.array_equal(d_cur.cpu().numpy(), w_new)
        assert np.array_equal(K.cpu().numpy(), w_K) and np.array_equal(nodes.cpu().numpy(), w_nodes)
        assert np.array_equal(changed.cpu().numpy().astype(bool), w_changed)


def test_closed_loop_reports_the_status_of_its_search():
    """A job whose re-allocation factor is not positive (T_j - R_j delta <= 0) raises a status bit in every fitness
    call of the search; the simulator tick that follows on the same workspace must not wipe it."""
    import paper_2008_12260_amd as px
    from paper_2008_12260_amd import closed_loop
    wl = W.make("tiny", current="fair")
    c = wl.cfg
    jp = wl.job_params.copy()
    jp[W.PARAM_INDEX["age_T"], 1] = 10.0
    jp[W.PARAM_INDEX["restarts_R"], 1] = 3.0
    seen = []
    closed_loop.run(jp, wl.m_grid, wl.fair_share, wl.node_capacity, np.full(c.J, 1e9), W.noise_scale_schedule(wl.param("phi")),
                    wl.current_alloc, P=32, Gs=c.Gs, generations=3, intervals=2, seed=5,
                    on_interval=lambda state, rec: seen.append(rec["status"]))
    assert seen == [px.PX_ST_BAD_RESTART] * 2


def test_closed_loop_is_checked_interval_by_interval():
    """The scheduling loop of paper_2008_12260_amd.closed_loop on the testbed-shaped workload: every interval's
    decision and tick are recomputed by the CPU checker from the inputs the loop used."""
    import oracle as O
    from paper_2008_12260_amd import closed_loop
    wl = W.make("physical", current="fair")
    c = wl.cfg
    target = np.full(c.J, 3.0e5)
    phi_of = W.noise_scale_schedule(wl.param("phi"))
    seen = []

    def check(state, rec):
        jp = wl.job_params.copy()
        jp[W.PARAM_INDEX["phi"]] = rec["phi"]
        both = np.stack([rec["alloc"], rec["previous_alloc"]])
        ref = O.fitness(both, jp, wl.m_grid, wl.fair_share, rec["previous_alloc"], wl.node_capacity, c.p, c.delta, c.Gs)
        assert rec["status"] == 0 and ref["violations"][0] == 0                       # the applied matrix is feasible
        assert abs(ref["fitness"][0] - rec["best_fitness"]) <= 1e-12 * abs(ref["fitness"][0])
        assert ref["fitness"][0] >= ref["fitness"][1] * (1 - 1e-12)                   # never worse than staying put
        changed = (rec["alloc"] != rec["previous_alloc"]).any(1) & (rec["previous_alloc"].sum(1) > 0)
        assert np.array_equal(changed, rec["changed"])              # what pollux_apply_best reported
        g, new, fin = LP.sim_tick(jp, wl.m_grid, c.Gs, rec["alloc"].sum(1), (rec["alloc"] > 0).sum(1), changed,
                                  rec["progress_before"], target, 60.0, 30.0)
        assert rel_err(rec["goodput"], g).max() <= RTOL and rel_err(rec["progress"], new).max() <= RTOL
        seen.append((rec["best_fitness"], int(rec["alloc"].sum())))

    kw = dict(P=128, Gs=c.Gs, p=c.p, delta=c.delta, generations=8, intervals=6, seed=7, on_interval=check)
    state = closed_loop.run(wl.job_params, wl.m_grid, wl.fair_share, wl.node_capacity, target, phi_of, wl.current_alloc, **kw)
    assert len(seen) == 6 and state.interval == 6
    assert np.all(state.progress > 0)
    assert seen[-1][1] >= seen[0][1]                            # the search hands out GPUs the fair share left idle
    # deterministic: the same run again ends in the same state; memoised or not makes no difference
    again = closed_loop.run(wl.job_params, wl.m_grid, wl.fair_share, wl.node_capacity, target, phi_of, wl.current_alloc,
                            **{**kw, "on_interval": None, "memoise": False})
    assert np.array_equal(again.alloc, state.alloc) and np.array_equal(again.progress, state.progress)
