"""GPU parity of pollux_ga_step against the CPU oracle: bit-exact matrices."""
import numpy as np
import pytest

import oracle as O
import workloads as W
from parity import run_oracle

pytestmark = pytest.mark.gpu
SEED = 0x2008_1226_0000_0001


def gpu_call(wl, P=None):
    import paper_2008_12260_amd as px
    c = wl.cfg
    return px.FitnessCall(c.P if P is None else P, c.J, c.N, c.Gm, c.Gs, wl.job_params, wl.m_grid, wl.fair_share,
                          wl.current_alloc, wl.node_capacity, p=c.p, delta=c.delta)


@pytest.mark.parametrize("name,mut", [("tiny", 1 << 29), ("physical", 1 << 29), ("physical", 0xFFFFFFFF), ("mid", 1 << 29)])
def test_single_step_matches_oracle(name, mut):
    import torch
    wl = W.make(name)
    c = wl.cfg
    fit = run_oracle(wl)["fitness"]
    call = gpu_call(wl)
    parents = torch.as_tensor(wl.population).cuda()
    children = torch.empty_like(parents)
    dfit = torch.as_tensor(fit).cuda()
    for gen in (0, 5):
        call.ga_step(parents, children, SEED, gen, c.P // 2, mut, fitness=dfit)
        want = O.ga_step(wl.population, fit, wl.node_capacity, SEED, gen, c.P // 2, mut)
        assert np.array_equal(children.cpu().numpy(), want)


@pytest.mark.parametrize("shape", [
    dict(P=4, J=1, N=1, cap=2, Gm=2, Gs=1),
    dict(P=7, J=5, N=3, cap=1, Gm=2, Gs=1),
    dict(P=6, J=300, N=70, cap=2, Gm=2, Gs=1),
    dict(P=5, J=9, N=300, cap=3, Gm=2, Gs=1),
    dict(P=6, J=150, N=48, cap=2, Gm=2, Gs=1),       # short rows: the unchanged ones are copied four to a wavefront load
    dict(P=9, J=33, N=64, cap=1, Gm=2, Gs=1),
])
def test_ragged_shapes_and_heavy_repair(shape):
    import torch
    cfg = W.custom("ga_ragged", **shape)
    wl = W.make(cfg)
    rng = np.random.default_rng(3)
    pop = wl.population + (rng.uniform(size=wl.population.shape) < 0.3)      # overload nodes, spread jobs
    pop = pop.astype(np.int32)
    fit = rng.choice([0.5, 0.7, -2.0, 1.0], cfg.P)                           # ties in the ranking
    call = gpu_call(wl)
    parents = torch.as_tensor(pop).cuda()
    children = torch.empty_like(parents)
    for elite in (1, cfg.P // 2, cfg.P):
        call.ga_step(parents, children, SEED, 9, elite, 1 << 31, fitness=torch.as_tensor(fit).cuda())
        want = O.ga_step(pop, fit, wl.node_capacity, SEED, 9, elite, 1 << 31)
        assert np.array_equal(children.cpu().numpy(), want)


@pytest.mark.parametrize("name,gens", [("physical", 30), ("mid", 40)])
def test_search_loop_matches_oracle_every_generation(name, gens):
    """fitness -> step -> fitness ... on both sides independently; matrices compared at every generation."""
    import torch
    wl = W.make(name)
    c = wl.cfg
    call = gpu_call(wl)
    a = torch.as_tensor(wl.population).cuda()
    b = torch.empty_like(a)
    host = wl.population
    mut = 1 << 29          # 1/8 per job
    for gen in range(gens):
        call.run(a, outputs="fitness")
        call.ga_step(a, b, SEED, gen, c.P // 2, mut)
        f = run_oracle(wl, population=host)["fitness"]
        host = O.ga_step(host, f, wl.node_capacity, SEED, gen, c.P // 2, mut)
        a, b = b, a
        got = a.cpu().numpy()
        assert np.array_equal(got, host), f"generation {gen}: {np.argwhere((got != host).any(axis=(1, 2))).ravel()[:8]}"
    # the search made progress and kept feasibility
    f_end = run_oracle(wl, population=host)
    assert f_end["fitness"].max() >= run_oracle(wl)["fitness"].max()
    assert np.all(f_end["violations"][c.P // 2:] == 0)


def test_rejects_aliasing_and_bad_elite():
    import torch
    import paper_2008_12260_amd as px
    wl = W.make("tiny")
    call = gpu_call(wl)
    a = torch.as_tensor(wl.population).cuda()
    with pytest.raises(px.PolluxError):
        call.ga_step(a, a, SEED, 0, 8, 0)
    with pytest.raises(px.PolluxError):
        call.ga_step(a, torch.empty_like(a), SEED, 0, 0, 0)
    with pytest.raises(px.PolluxError):
        call.ga_step(a, torch.empty_like(a), SEED, 0, 17, 0)


def test_large_config_one_generation_bit_exact():
    """One search step on the full 4096 x 1000 x 256 population against the oracle (all 4.19 GB compared)."""
    import torch
    cfg = W.CONFIGS["large"]
    wl = W.make(cfg, with_population=False)
    pop = W.candidates(cfg, 0, cfg.P)
    rng = np.random.default_rng(8)
    fit = rng.uniform(0.2, 1.0, cfg.P)
    fit[::20] = -3.0
    fit[5] = fit[6] = fit[4000]                       # ties in the ranking
    call = gpu_call(wl)
    parents = torch.from_numpy(pop).cuda()
    children = torch.empty_like(parents)
    call.ga_step(parents, children, SEED, 3, cfg.P // 2, 1 << 29, fitness=torch.as_tensor(fit).cuda())
    got = children.cpu().numpy()
    del parents, children
    want = O.ga_step(pop, fit, wl.node_capacity, SEED, 3, cfg.P // 2, 1 << 29)
    for lo in range(0, cfg.P, 256):
        assert np.array_equal(got[lo:lo + 256], want[lo:lo + 256]), f"children {lo}..{lo + 255}"


@pytest.mark.parametrize("name", ["tiny", "physical", "mid"])
def test_in_place_step_matches_oracle(name):
    """PX_GA_IN_PLACE: children overwrite the slots of the candidates that did not survive."""
    import torch
    import paper_2008_12260_amd as px
    wl = W.make(name)
    c = wl.cfg
    fit = run_oracle(wl)["fitness"]
    call = gpu_call(wl)
    for elite in (1, c.P // 2, c.P):
        pop = torch.as_tensor(wl.population).cuda()
        call.ga_step(pop, pop, SEED, 4, elite, 1 << 29, fitness=torch.as_tensor(fit).cuda(), flags=px.PX_GA_IN_PLACE)
        want = O.ga_step(wl.population, fit, wl.node_capacity, SEED, 4, elite, 1 << 29, flags=O.GA_IN_PLACE)
        assert np.array_equal(pop.cpu().numpy(), want)


def test_in_place_search_loop_matches_oracle_every_generation():
    import torch
    import paper_2008_12260_amd as px
    wl = W.make("physical")
    c = wl.cfg
    call = gpu_call(wl)
    host = wl.population.copy()
    dev = torch.as_tensor(host).cuda()
    for gen in range(25):
        ref = run_oracle(wl, population=host)
        call.run(dev)
        got = call.results()
        assert np.array_equal(got["best_m"], ref["best_m"]) and np.array_equal(got["violations"], ref["violations"])
        # the step is driven by the oracle's fitness on both sides, so that one ulp never forks the two searches
        host = O.ga_step(host, ref["fitness"], wl.node_capacity, SEED, gen, c.P // 2, (1 << 32) // c.J, flags=O.GA_IN_PLACE)
        call.ga_step(dev, dev, SEED, gen, c.P // 2, (1 << 32) // c.J, fitness=torch.as_tensor(ref["fitness"]).cuda(),
                     flags=px.PX_GA_IN_PLACE)
        assert np.array_equal(dev.cpu().numpy(), host), f"generation {gen}"


def test_in_place_flag_needs_the_same_buffer_and_unknown_flags_are_rejected():
    import torch
    import paper_2008_12260_amd as px
    wl = W.make("tiny")
    call = gpu_call(wl)
    a = torch.as_tensor(wl.population).cuda()
    with pytest.raises(px.PolluxError):
        call.ga_step(a, torch.empty_like(a), SEED, 0, 8, 0, flags=px.PX_GA_IN_PLACE)
    with pytest.raises(px.PolluxError):
        call.ga_step(a, torch.empty_like(a), SEED, 0, 8, 0, flags=2)


@pytest.mark.parametrize("name", ["tiny", "physical", "mid"])
def test_job_gpu_limits_match_oracle(name):
    """pollux_ga_params.job_gpu_cap: rows of children are cut back to the job's limit before the repairs."""
    import torch
    import paper_2008_12260_amd as px
    wl = W.make(name)
    c = wl.cfg
    fit = run_oracle(wl)["fitness"]
    limits = np.random.default_rng(9).integers(0, 6, c.J).astype(np.int32)
    limits[::7] = 10**6
    assert (wl.population.sum(2) > limits[None]).any()
    call = gpu_call(wl)
    dl = torch.as_tensor(limits).cuda()
    dfit = torch.as_tensor(fit).cuda()
    parents = torch.as_tensor(wl.population).cuda()
    children = torch.empty_like(parents)
    call.ga_step(parents, children, SEED, 2, c.P // 2, 1 << 30, fitness=dfit, job_gpu_cap=dl)
    want = O.ga_step(wl.population, fit, wl.node_capacity, SEED, 2, c.P // 2, 1 << 30, job_gpu_cap=limits)
    assert np.array_equal(children.cpu().numpy(), want)
    call.ga_step(parents, parents, SEED, 2, c.P // 2, 1 << 30, fitness=dfit, job_gpu_cap=dl, flags=px.PX_GA_IN_PLACE)
    want = O.ga_step(wl.population, fit, wl.node_capacity, SEED, 2, c.P // 2, 1 << 30, job_gpu_cap=limits, flags=O.GA_IN_PLACE)
    assert np.array_equal(parents.cpu().numpy(), want)


def test_job_gpu_limits_on_long_unaligned_rows():
    import torch
    cfg = W.custom("ga_limits", P=6, J=9, N=300, cap=3, Gm=2, Gs=1)
    wl = W.make(cfg)
    rng = np.random.default_rng(4)
    pop = (wl.population + (rng.uniform(size=wl.population.shape) < 0.2)).astype(np.int32)
    fit = rng.uniform(size=cfg.P)
    limits = rng.integers(0, 30, cfg.J).astype(np.int32)
    call = gpu_call(wl)
    parents = torch.as_tensor(pop).cuda()
    children = torch.empty_like(parents)
    call.ga_step(parents, children, SEED, 1, 2, 1 << 31, fitness=torch.as_tensor(fit).cuda(), job_gpu_cap=torch.as_tensor(limits).cuda())
    want = O.ga_step(pop, fit, wl.node_capacity, SEED, 1, 2, 1 << 31, job_gpu_cap=limits)
    assert np.array_equal(children.cpu().numpy(), want)


def test_large_config_one_generation_in_place_bit_exact():
    """The search step as bench.py runs it (in place, 2048 children formed) on the full population."""
    import torch
    import paper_2008_12260_amd as px
    cfg = W.CONFIGS["large"]
    wl = W.make(cfg, with_population=False)
    pop = W.candidates(cfg, 0, cfg.P)
    rng = np.random.default_rng(18)
    fit = rng.uniform(0.2, 1.0, cfg.P)
    fit[::20] = -3.0
    call = gpu_call(wl)
    dev = torch.from_numpy(pop).cuda()
    call.ga_step(dev, dev, SEED, 7, cfg.P // 2, (1 << 32) // cfg.J, fitness=torch.as_tensor(fit).cuda(),
                 flags=px.PX_GA_IN_PLACE)
    got = dev.cpu().numpy()
    del dev
    want = O.ga_step(pop, fit, wl.node_capacity, SEED, 7, cfg.P // 2, (1 << 32) // cfg.J, flags=O.GA_IN_PLACE)
    for lo in range(0, cfg.P, 256):
        assert np.array_equal(got[lo:lo + 256], want[lo:lo + 256]), f"candidates {lo}..{lo + 255}"


@pytest.mark.parametrize("flags", [0, 4])
def test_search_loop_in_the_benchmark_shape_matches_oracle_every_generation(flags):
    """The loop as bench.py runs it on the 64 x 8 cluster: step in place, job tables kept after the first
    generation, the library's own fitness driving its own step, plain and memoised (flags = 4); the checker
    runs its own independent loop.  Matrices, elected points and violation counts are compared at every one of
    100 generations."""
    import torch
    import paper_2008_12260_amd as px
    wl = W.make("mid")
    c = wl.cfg
    call = px.FitnessCall(c.P, c.J, c.N, c.Gm, c.Gs, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc,
                          wl.node_capacity, p=c.p, delta=c.delta, flags=flags)
    host = wl.population.copy()
    dev = torch.as_tensor(host).cuda()
    mut = (1 << 32) // c.J
    first_best = None
    for gen in range(100):
        call.run(dev, outputs="argmax", keep_job_tables=gen > 0)
        ref = run_oracle(wl, population=host)
        if gen % 10 == 0 or gen == 99:
            got = call.results()
            assert got["status"] == ref["status"] == 0
            assert np.array_equal(got["best_m"], ref["best_m"]) and np.array_equal(got["best_s"], ref["best_s"]), gen
            assert np.array_equal(got["violations"], ref["violations"]), gen
            err = np.abs(got["fitness"] - ref["fitness"]) / np.where(ref["fitness"] == 0, 1.0, np.abs(ref["fitness"]))
            assert err.max() <= 1e-12, gen
        first_best = ref["fitness"].max() if first_best is None else first_best
        call.ga_step(dev, dev, SEED, gen, c.P // 2, mut, flags=px.PX_GA_IN_PLACE)
        host = O.ga_step(host, ref["fitness"], wl.node_capacity, SEED, gen, c.P // 2, mut, flags=O.GA_IN_PLACE)
        got = dev.cpu().numpy()
        assert np.array_equal(got, host), f"generation {gen}: {np.argwhere((got != host).any(axis=(1, 2))).ravel()[:8]}"
    assert run_oracle(wl, population=host)["fitness"].max() >= first_best


def test_step_with_zero_grid_dims_between_fitness_calls_that_keep_their_tables():
    """pollux_ga_step reads P, J, N only: called through the C ABI with Gm = Gs = 0 on the workspace of a search
    whose fitness calls keep their job tables, it must leave those tables alone."""
    import ctypes
    import torch
    import paper_2008_12260_amd as px
    wl = W.make("physical")
    c = wl.cfg
    call = px.FitnessCall(c.P, c.J, c.N, c.Gm, c.Gs, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc,
                          wl.node_capacity, p=c.p, delta=c.delta)
    dev = torch.as_tensor(wl.population).cuda()
    call.run(dev)
    first = call.results()
    bare = px.Dims(c.P, c.J, c.N, 0, 0, 0, 0)
    ga = px.GaParams(SEED, 0, c.P // 2, (1 << 32) // c.J, px.PX_GA_IN_PLACE, None)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    ptr = lambda t: ctypes.c_void_p(t.data_ptr())
    rc = px.lib().pollux_ga_step(ctypes.byref(bare), ptr(dev), ptr(call.fitness), ptr(call.node_capacity), ctypes.byref(ga),
                                 ptr(call.workspace), call.workspace.numel(), ptr(dev), stream)
    assert rc == px.PX_OK
    want = O.ga_step(wl.population, first["fitness"], wl.node_capacity, SEED, 0, c.P // 2, (1 << 32) // c.J, flags=O.GA_IN_PLACE)
    assert np.array_equal(dev.cpu().numpy(), want)
    call.run(dev, keep_job_tables=True)
    kept = call.results()
    ref = run_oracle(wl, population=want)
    assert np.array_equal(kept["best_m"], ref["best_m"]) and np.array_equal(kept["best_s"], ref["best_s"])
    assert np.allclose(kept["fitness"], ref["fitness"], rtol=1e-12, atol=0.0)
    assert np.allclose(kept["best_goodput"], ref["best_goodput"], rtol=1e-12, atol=0.0)


# ---- pollux_generation: the step in place followed by the fitness of the children only ------------------------

def generation_loop(wl, gens, flags=0, precision=0, elite=None, mut=None, check_every=1, P=None, inherit=False, pop=None):
    """Both sides run fitness once and then `gens` generations; every output array is compared each time."""
    import torch
    import paper_2008_12260_amd as px
    from parity import compare
    c = wl.cfg
    pop0 = (wl.population if pop is None else pop) if P is None else wl.population[:P]
    P = pop0.shape[0]
    elite = P // 2 if elite is None else elite
    mut = (1 << 32) // c.J if mut is None else mut
    if inherit and (flags & px.PX_FLAG_MEMOISE):
        flags |= px.PX_FLAG_PAIR_RESULTS           # a memoised call keeps its per-pair results only on request
    call = px.FitnessCall(P, c.J, c.N, c.Gm, c.Gs, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc,
                          wl.node_capacity, p=c.p, delta=c.delta, flags=flags, precision=precision)
    dev = torch.as_tensor(pop0).cuda()
    call.run(dev)
    host = pop0.copy()
    ref = run_oracle(wl, population=host)
    for gen in range(gens):
        call.generation(dev, SEED, gen, elite, mut, inherit_rows=inherit)
        host, ref = O.generation(host, ref["fitness"], wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc,
                                 wl.node_capacity, c.p, c.delta, c.Gs, SEED, gen, elite, mut)
        got_pop = dev.cpu().numpy()
        assert np.array_equal(got_pop, host), f"generation {gen}: {np.argwhere((got_pop != host).any(axis=(1, 2))).ravel()[:8]}"
        if gen % check_every == 0 or gen == gens - 1:
            got = call.results()
            if precision == 0:
                assert compare(wl, got, ref, population=host) == 0, gen
            else:
                assert np.array_equal(got["violations"], ref["violations"])
                err = np.abs(got["fitness"] - ref["fitness"]) / np.where(ref["fitness"] == 0, 1.0, np.abs(ref["fitness"]))
                assert err.max() <= 1e-5, gen
    return call, dev, host


@pytest.mark.parametrize("inherit", [False, True])
@pytest.mark.parametrize("flags", [0, 4])
def test_generation_call_matches_oracle_every_generation_on_the_mid_configuration(flags, inherit):
    """60 generations of pollux_generation (survivors keep their results, children are swept, or with
    PX_GA_INHERIT_ROWS only their changed rows) against the checker's step + full evaluation; matrices every
    generation, every fitness output every tenth."""
    import paper_2008_12260_amd as px
    wl = W.make("mid")
    call, dev, host = generation_loop(wl, 60, flags=flags, check_every=10, inherit=inherit)
    # and a full evaluation of the final population by the library gives bit for bit what the incremental calls left
    kept = call.results()
    call.run(dev, keep_job_tables=True)
    full = call.results()
    for k in ("fitness", "best_m", "best_s", "best_goodput", "speedup", "violations"):
        assert np.array_equal(kept[k], full[k], equal_nan=True), k


@pytest.mark.parametrize("shape,elite", [
    (dict(P=7, J=5, N=3, cap=2, Gm=5, Gs=3), 3),
    (dict(P=9, J=13, N=67, cap=2, Gm=70, Gs=5), 1),           # all but one candidate replaced each generation
    (dict(P=37, J=11, N=64, cap=8, Gm=64, Gs=16), 20),        # rows read four to a load, odd count of children
    (dict(P=21, J=9, N=256, cap=4, Gm=64, Gs=32), 10),        # one row per load, whole groups of batch sizes
    (dict(P=530, J=200, N=64, cap=8, Gm=64, Gs=16), 263),     # several candidates per wavefront
    (dict(P=40, J=70, N=128, cap=2, Gm=20, Gs=6), 40),        # nothing to form: every candidate survives
    (dict(P=6, J=40, N=9, cap=40, Gm=33, Gs=5), 2),           # rows beyond the tables
])
@pytest.mark.parametrize("inherit", [False, True])
@pytest.mark.parametrize("flags", [0, 4, 16])
def test_generation_call_on_ragged_shapes(shape, elite, flags, inherit):
    cfg = W.custom("gen_ragged", **shape)
    wl = W.make(cfg)
    if flags == 16:
        wl = W.sampled(wl)
        import torch
        import paper_2008_12260_amd as px
        c = wl.cfg
        call = px.FitnessCall(c.P, c.J, c.N, c.Gm, c.Gs, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc,
                              wl.node_capacity, p=c.p, delta=c.delta, flags=16)
        dev = torch.as_tensor(wl.population).cuda()
        call.run(dev)
        host, ref = wl.population.copy(), run_oracle(wl, flags=16)
        for gen in range(3):
            call.generation(dev, SEED, gen, elite, 1 << 30, inherit_rows=inherit)
            host, ref = O.generation(host, ref["fitness"], wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc,
                                     wl.node_capacity, c.p, c.delta, c.Gs, SEED, gen, elite, 1 << 30, flags=16)
            assert np.array_equal(dev.cpu().numpy(), host)
            got = call.results()
            assert np.array_equal(got["best_m"], ref["best_m"]) and np.array_equal(got["best_s"], ref["best_s"])
            assert np.allclose(got["fitness"], ref["fitness"], rtol=1e-12, atol=0.0, equal_nan=True)
        return
    generation_loop(wl, 4, flags=flags, elite=elite, mut=1 << 30, inherit=inherit)


def test_generation_call_in_fp32_and_its_argument_checks():
    import torch
    import paper_2008_12260_amd as px
    wl = W.make("physical")
    generation_loop(wl, 5, precision=1)
    generation_loop(wl, 5, precision=1, inherit=True)
    c = wl.cfg
    call = gpu_call(wl)
    dev = torch.as_tensor(wl.population).cuda()
    call.run(dev)
    ga = px.GaParams(SEED, 0, c.P // 2, 0, 0, None)          # not in place
    with pytest.raises(px.PolluxError):
        px.pollux_generation(call.dims, dev, call.job_params, call.m_grid, call.fair_share, call.current_alloc,
                             call.node_capacity, c.p, c.delta, ga, call.workspace, call.fitness, call.best_m, call.best_s)
    ga = px.GaParams(SEED, 0, c.P + 1, 0, px.PX_GA_IN_PLACE, None)
    with pytest.raises(px.PolluxError):
        px.pollux_generation(call.dims, dev, call.job_params, call.m_grid, call.fair_share, call.current_alloc,
                             call.node_capacity, c.p, c.delta, ga, call.workspace, call.fitness, call.best_m, call.best_s)


@pytest.mark.parametrize("inherit", [False, True])
def test_generation_call_on_the_large_configuration(inherit):
    """The headline shape: one full evaluation, then two generations that sweep the 2048 children only; the oracle
    recomputes the children of the last generation (the slots that were rewritten) and a sample of survivors."""
    import torch
    import paper_2008_12260_amd as px
    from parity import compare
    cfg = W.CONFIGS["large"]
    wl = W.make(cfg, with_population=False)
    pop = W.candidates(cfg, 0, cfg.P)
    call = px.FitnessCall(cfg.P, cfg.J, cfg.N, cfg.Gm, cfg.Gs, wl.job_params, wl.m_grid, wl.fair_share,
                          wl.current_alloc, wl.node_capacity, p=cfg.p, delta=cfg.delta)
    dev = torch.from_numpy(pop).cuda()
    call.run(dev)
    host = pop
    fit = call.results()["fitness"]
    mut = (1 << 32) // cfg.J
    for gen in range(2):
        before = call.results()
        call.generation(dev, SEED, gen, cfg.P // 2, mut, inherit_rows=inherit)
        host = O.ga_step(host, before["fitness"], wl.node_capacity, SEED, gen, cfg.P // 2, mut, flags=O.GA_IN_PLACE)
        order = O.rank(before["fitness"])
        got = call.results()
        survivors = order[:cfg.P // 2]
        for k in ("fitness", "best_m", "best_s", "best_goodput", "speedup", "violations"):
            assert np.array_equal(got[k][survivors], before[k][survivors], equal_nan=True), k
    got_pop = dev.cpu().numpy()
    for lo in range(0, cfg.P, 256):
        assert np.array_equal(got_pop[lo:lo + 256], host[lo:lo + 256]), f"candidates {lo}..{lo + 255}"
    idx = np.concatenate([order[cfg.P // 2:][::16], order[:cfg.P // 2][::64]])       # 128 children, 32 survivors
    sub = host[idx]
    ref = run_oracle(wl, population=sub)
    gs = {k: (v[idx] if isinstance(v, np.ndarray) else v) for k, v in got.items()}
    assert compare(wl, gs, ref, population=sub) == 0


@pytest.mark.parametrize("inherit", [False, True])
@pytest.mark.parametrize("flags", [0, 4])
@pytest.mark.parametrize("shape", [None, dict(P=12, J=70, N=128, cap=2, Gm=20, Gs=6)])
def test_generations_that_write_fitness_only(flags, shape, inherit):
    """A search needs only fitness: with best_m and best_s left out (NULL) the generations form the same matrices and
    the same fitness and violation counts, and nothing is written per pair."""
    import torch
    import paper_2008_12260_amd as px
    wl = W.make("physical") if shape is None else W.make(W.custom("fitness_only", **shape))
    c = wl.cfg
    if inherit and flags:
        flags |= px.PX_FLAG_PAIR_RESULTS
    calls, pops = [], []
    for outputs in ("all", "fitness"):
        call = px.FitnessCall(c.P, c.J, c.N, c.Gm, c.Gs, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc,
                              wl.node_capacity, p=c.p, delta=c.delta, flags=flags)
        for t in (call.best_m, call.best_s):
            t.fill_(-7)
        call.best_goodput.fill_(-7.0)
        call.speedup.fill_(-7.0)
        dev = torch.as_tensor(wl.population).cuda()
        call.run(dev, outputs=outputs)
        for gen in range(20):
            call.generation(dev, SEED, gen, c.P // 2, (1 << 32) // c.J, outputs=outputs, inherit_rows=inherit)
        calls.append(call.results())
        pops.append(dev.cpu().numpy())
    assert np.array_equal(pops[0], pops[1])
    for k in ("fitness", "violations"):
        assert np.array_equal(calls[0][k], calls[1][k], equal_nan=True), k
    assert calls[0]["status"] == calls[1]["status"]
    for k in ("best_m", "best_s", "best_goodput", "speedup"):
        assert np.all(calls[1][k] == -7), k
    assert np.all(calls[0]["best_s"] >= -1)


@pytest.mark.parametrize("flags", [0, 4])
def test_inherited_rows_with_children_that_cannot_be_taken_for_granted(flags):
    """PX_GA_INHERIT_ROWS on populations whose children the step flags: matrices dense enough to overflow the
    per-node lists on chip (the column path of the repairs), parents with negative entries; and a node without
    capacity.  Such children are evaluated in full; everything must equal the checker's step + full evaluation,
    violation counts and the status word included."""
    cfg = W.custom("odd_children", P=24, J=40, N=64, cap=4, Gm=64, Gs=16)
    wl = W.make(cfg)
    rng = np.random.default_rng(11)
    dense = wl.population.copy()
    dense[::3] = (rng.random(dense[::3].shape) < 0.4).astype(np.int32) * rng.integers(1, 3, dense[::3].shape, dtype=np.int32)
    assert (dense[0] > 0).sum() > 512                                   # more entries than the lists of this shape hold
    generation_loop(wl, 4, flags=flags, mut=1 << 29, inherit=True, pop=dense)
    negative = wl.population.copy()
    negative[:, ::5, 3] = -1            # in every candidate, so that the (accumulating) status word and the checker's agree
    generation_loop(wl, 4, flags=flags, mut=1 << 29, inherit=True, pop=negative)
    import dataclasses
    cap = wl.node_capacity.copy()
    cap[5] = 0
    generation_loop(dataclasses.replace(wl, node_capacity=cap), 4, flags=flags, mut=1 << 29, inherit=True)
