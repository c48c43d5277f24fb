"""The search loop recorded into a HIP graph: every replay must give what the same launches give when issued one by one.

The library's calls allocate nothing, clear their counters with kernels of their own and take the caller's stream,
so a caller may record them; this is the check that doing so changes nothing.  The recorded generation numbers are
fixed in the graph, so a replay repeats them (on the population the replay before it left): the eager run repeats
them too."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu
SEED = 0x2008_1226_0000_0003


@pytest.mark.parametrize("inherit", [False, True])
def test_replays_of_a_recorded_search_loop_match_the_same_launches_issued_one_by_one(inherit):
    import torch
    import paper_2008_12260_amd as px
    cfg = W.custom("graph", P=96, J=40, N=24, cap=4, Gm=64, Gs=16)
    wl = W.make(cfg)
    mut = (1 << 32) // 8
    gens, replays = (3, 4, 5), 4

    def make_call():
        return px.FitnessCall(cfg.P, cfg.J, cfg.N, cfg.Gm, cfg.Gs, wl.job_params, wl.m_grid, wl.fair_share,
                              wl.current_alloc, wl.node_capacity, p=cfg.p, delta=cfg.delta)

    def snapshot(call, pop):
        torch.cuda.synchronize()
        r = call.results()
        return pop.cpu().numpy().copy(), {k: np.array(r[k], copy=True) for k in ("fitness", "best_m", "best_s", "best_goodput", "speedup")}

    # one by one
    call = make_call()
    pop = torch.as_tensor(wl.population).cuda()
    call.run(pop)
    want = []
    for _ in range(replays + 1):                      # the recording pass itself runs nothing: one more round below makes up for it
        for g in gens:
            call.generation(pop, SEED, g, cfg.P // 2, mut, inherit_rows=inherit)
        want.append(snapshot(call, pop))

    # recorded
    call = make_call()
    pop = torch.as_tensor(wl.population).cuda()
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        call.run(pop, stream=s)
        for g in gens:                                # first use of every kernel outside the recording
            call.generation(pop, SEED, g, cfg.P // 2, mut, stream=s, inherit_rows=inherit)
        s.synchronize()
        got = [snapshot(call, pop)]
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=s):
            for g in gens:
                call.generation(pop, SEED, g, cfg.P // 2, mut, stream=s, inherit_rows=inherit)
        for _ in range(replays):
            graph.replay()
            got.append(snapshot(call, pop))
            # the program's own work between replays: an eager fitness call on another population, another workspace
            other = make_call()
            other.run(torch.as_tensor(wl.population).cuda())
            torch.cuda.synchronize()
    for k, ((wp, wr), (gp, gr)) in enumerate(zip(want, got)):
        assert np.array_equal(wp, gp), f"population after round {k}"
        for name in wr:
            assert np.array_equal(wr[name], gr[name], equal_nan=True), (k, name)
