"""pollux_fitness_static (the entry point for callers that cannot allocate device memory) against pollux_fitness.

Two calls in a row through the C ABI, the second on a smaller problem, each compared with what pollux_fitness
gives for the same inputs: the same kernels run on the library's own scratch array, so every output must be
bit-identical, and nothing the first call left in the array may leak into the second."""
import ctypes

import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu

OUTPUTS = ("fitness", "best_m", "best_s", "best_goodput", "speedup", "violations")


def both_ways(wl, population, flags=0, precision=0):
    """(results of pollux_fitness, results of pollux_fitness_static) for one workload, as dicts of numpy arrays."""
    import torch
    import paper_2008_12260_amd as px
    c = wl.cfg
    P = population.shape[0]
    call = px.FitnessCall(P, c.J, c.N, c.Gm, c.Gs, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc,
                          wl.node_capacity, p=c.p, delta=c.delta, flags=flags, precision=precision)
    dpop = torch.as_tensor(population, dtype=torch.int32).contiguous().cuda()
    call.run(dpop)
    want = call.results()
    # outputs of the second way: allocated here, by the caller; the call itself gets no workspace
    out = dict(fitness=torch.full((P,), -7.0, dtype=torch.float64, device="cuda"),
               best_m=torch.full((P, c.J), -7, dtype=torch.int32, device="cuda"),
               best_s=torch.full((P, c.J), -7, dtype=torch.int32, device="cuda"),
               best_goodput=torch.full((P, c.J), -7.0, dtype=torch.float64, device="cuda"),
               speedup=torch.full((P, c.J), -7.0, dtype=torch.float64, device="cuda"),
               violations=torch.full((P,), -7, dtype=torch.int32, device="cuda"))
    status = torch.full((1,), -7, dtype=torch.int32, device="cuda")
    torch.cuda.synchronize()
    px.pollux_fitness_static(call.dims, dpop, call.job_params, call.m_grid, call.fair_share, call.current_alloc,
                             call.node_capacity, call.p, call.delta, out["fitness"], out["best_m"], out["best_s"],
                             out["best_goodput"], out["speedup"], out["violations"], status)
    torch.cuda.synchronize()
    got = {k: v.cpu().numpy() for k, v in out.items()}
    got["status"] = int(status.item())
    return want, got


def assert_same(want, got):
    assert got["status"] == want["status"]
    for k in OUTPUTS:
        assert np.array_equal(got[k], want[k], equal_nan=True), k


def test_two_calls_in_a_row_the_second_on_a_smaller_problem():
    import paper_2008_12260_amd as px
    big = W.make("mid")                       # 46 MiB of scratch: most of the array
    assert px.workspace_size(px.Dims(big.cfg.P, big.cfg.J, big.cfg.N, big.cfg.Gm, big.cfg.Gs, 0, 0)) <= px.STATIC_SCRATCH_BYTES
    spoiled = big.population.copy()
    spoiled[::7] *= 3                         # many nodes over capacity: the per-node counters are exercised
    want, got = both_ways(big, spoiled)
    assert want["violations"].max() > 0
    assert_same(want, got)
    small = W.make("physical")                # smaller in every dimension; other jobs, other grid
    jp = small.job_params.copy()
    jp[W.PARAM_INDEX["age_T"], 1] = 10.0      # a status bit that the first call did not raise
    jp[W.PARAM_INDEX["restarts_R"], 1] = 3.0
    small.job_params = jp
    want, got = both_ways(small, small.population)
    assert want["status"] == px.PX_ST_BAD_RESTART
    assert_same(want, got)
    tiny = W.make("tiny")
    for flags, precision in ((px.PX_FLAG_MEMOISE, 0), (0, 1)):
        want, got = both_ways(tiny, tiny.population, flags=flags, precision=precision)
        assert_same(want, got)


def test_a_problem_beyond_the_array_is_rejected_before_anything_runs():
    import torch
    import paper_2008_12260_amd as px
    d = px.Dims(4096, 1000, 256, 128, 32, 0, 0)
    assert px.workspace_size(d) > px.STATIC_SCRATCH_BYTES
    fake = ctypes.c_void_p(0x1000)            # never dereferenced: the size check comes first
    rc = px.lib().pollux_fitness_static(ctypes.byref(d), *([fake] * 6), -1.0, 30.0, *([fake] * 7), None)
    assert rc == px.PX_E_WORKSPACE
    assert torch.cuda.is_available()
