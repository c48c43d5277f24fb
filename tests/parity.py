"""Helpers of the GPU parity tests: run both sides on one workload and compare.

Tolerances (fp64 path): goodput, SPEEDUP and FITNESS within 1e-12 relative of
the oracle; (m*, s*), violation counts and the status word bit-exact.  A
differing (m*, s*) is accepted only when the oracle itself, re-evaluated in
extended precision, puts the two best distinct values closer than 1e-14
relative (a tie at fp64 resolution: the two sides evaluate the last pass of
Eq. 10 by different routes, a few units in the last place apart); such cases
are counted and returned.
"""
import numpy as np

import oracle as O

RTOL = 1e-12
TIE_GAP = 1e-14


def run_oracle(wl, population=None, p=None, delta=None, flags=0, current=None, job_params=None):
    c = wl.cfg
    return O.fitness(wl.population if population is None else population,
                     wl.job_params if job_params is None else job_params, wl.m_grid, wl.fair_share,
                     wl.current_alloc if current is None else current, wl.node_capacity,
                     c.p if p is None else p, c.delta if delta is None else delta, c.Gs, flags)


def run_gpu(wl, population=None, p=None, delta=None, flags=0, current=None, job_params=None, precision=0):
    import torch
    import paper_2008_12260_amd as px
    c = wl.cfg
    pop = wl.population if population is None else population
    P = pop.shape[0]
    call = px.FitnessCall(P, c.J, c.N, c.Gm, c.Gs, wl.job_params if job_params is None else job_params, wl.m_grid,
                          wl.fair_share, wl.current_alloc if current is None else current, wl.node_capacity,
                          p=c.p if p is None else p, delta=c.delta if delta is None else delta, flags=flags,
                          precision=precision)
    dpop = torch.as_tensor(pop, dtype=torch.int32).contiguous().cuda()
    call.run(dpop)
    return call.results()


def rel_err(got, want):
    got, want = np.asarray(got, np.float64), np.asarray(want, np.float64)
    both_nan = np.isnan(got) & np.isnan(want)
    same = (got == want) | both_nan
    denom = np.where(want == 0, 1.0, np.abs(want))
    err = np.where(same, 0.0, np.abs(got - want) / denom)
    err = np.where(np.isnan(err), np.inf, err)
    return err


def compare(wl, gpu, ref, population=None, rtol=RTOL, job_params=None, sampled=False):
    """Assert parity; return the number of sub-resolution ties in (m*, s*).

    sampled: the calls used the sampling argmax of Sec. 4.3 (the grid rows are total batch sizes); a differing
    choice is then accepted only when the GPU's point prices within TIE_GAP of the oracle's best."""
    c = wl.cfg
    pop = wl.population if population is None else population
    jp = wl.job_params if job_params is None else job_params
    assert gpu["status"] == ref["status"], (gpu["status"], ref["status"])
    assert np.array_equal(gpu["violations"], ref["violations"])
    mism = np.argwhere((gpu["best_m"] != ref["best_m"]) | (gpu["best_s"] != ref["best_s"]))
    ties = 0
    for cand, j in mism:
        K = int(pop[cand, j].sum())
        nodes = int((pop[cand, j] > 0).sum())
        jb = O.job_from_params(jp, j)
        gap = 0.0 if sampled else O.argmax_gap(jb, wl.m_grid[j], c.Gs, K, nodes)
        gm, gs = int(gpu["best_m"][cand, j]), int(gpu["best_s"][cand, j])
        assert gm > 0 and gs >= 0, f"pair ({cand},{j}): GPU found no point, oracle did"
        g_at, ok = O.goodput(jb, K, nodes, gm, gs)
        best = ref["best_goodput"][cand, j]
        assert ok and gap < TIE_GAP and abs(g_at - best) <= TIE_GAP * best, \
            f"pair ({cand},{j}) K={K} nodes={nodes}: GPU (m,s)=({gm},{gs}) oracle=({ref['best_m'][cand, j]}," \
            f"{ref['best_s'][cand, j]}) gap={gap:.3e} goodput at GPU point {g_at!r} vs best {best!r}"
        ties += 1
    for name in ("best_goodput", "speedup", "fitness"):
        e = rel_err(gpu[name], ref[name])
        worst = np.unravel_index(np.argmax(e), e.shape)
        assert e.max() <= rtol, f"{name}: rel err {e.max():.3e} at {worst}: {gpu[name][worst]!r} vs {ref[name][worst]!r}"
    return ties
