"""A scheduling loop on synthetic jobs, built from the library's calls only (Pollux, arXiv 2008.12260,
Sec. 4: every scheduling interval PolluxSched searches for a better allocation matrix, applies the best one,
and the jobs run on it until the next interval; Sec. 5.3: discrete-time simulation with a restart delay).

Per interval:
  1. the jobs' gradient noise scale phi_t is refreshed from their progress (the caller's `phi_of` function);
  2. the population search runs pollux_fitness once and then `generations` calls of pollux_generation (rows that a
     child holds unchanged inherit their parent's results) from a population seeded with the current allocation;
  3. pollux_apply_best takes the best candidate of the last evaluation, makes it the current allocation and
     marks the jobs whose row changed as re-allocated;
  4. pollux_sim_tick advances every job on its new allocation.

This module marshals arguments and copies results to the host for the caller's records; every step of the
method (the search, the choice of the best matrix, K / nodes / changed of its rows, the tick) runs in the
library's kernels.  It fails if the library is missing, like the rest of the package.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from . import (PX_FLAG_MEMOISE, PX_FLAG_PAIR_RESULTS, Dims, FitnessCall, PARAM_PHI, pollux_apply_best, pollux_sim_tick)


@dataclass
class LoopState:
    alloc: np.ndarray                 # int32 [J,N] current allocation
    progress: np.ndarray              # float64 [J]
    finished: np.ndarray              # bool [J]
    interval: int = 0
    history: list = field(default_factory=list)


def run(job_params, m_grid, fair_share, node_capacity, target, phi_of, alloc0, *, P=256, Gs=16, p=-1.0, delta=30.0,
        interval_s=60.0, restart_delay=30.0, generations=20, intervals=10, seed=1, memoise=True, on_interval=None):
    """Run `intervals` scheduling intervals; returns the final LoopState.

    phi_of(progress / target) -> phi_t per job (numpy, float64 [J]); on_interval(state, record) is called after
    every interval with a dict holding what was decided and measured (for tests and reports)."""
    import torch
    job_params = np.array(job_params, dtype=np.float64, copy=True)
    J, Gm = m_grid.shape
    N = len(node_capacity)
    dev = torch.device("cuda")
    state = LoopState(alloc=np.array(alloc0, dtype=np.int32, copy=True), progress=np.zeros(J), finished=np.zeros(J, bool))
    d_target = torch.as_tensor(np.asarray(target, np.float64)).to(dev)
    d_progress = torch.zeros(J, dtype=torch.float64, device=dev)
    d_goodput = torch.empty(J, dtype=torch.float64, device=dev)
    d_finished = torch.empty(J, dtype=torch.int32, device=dev)
    d_best = torch.empty(1, dtype=torch.int32, device=dev)
    d_K, d_nodes, d_changed = (torch.empty(J, dtype=torch.int32, device=dev) for _ in range(3))
    mut = max(1, (1 << 32) // J)
    for it in range(intervals):
        job_params[PARAM_PHI] = phi_of(np.minimum(state.progress / np.asarray(target, np.float64), 1.0))
        call = FitnessCall(P, J, N, Gm, Gs, job_params, m_grid, fair_share, state.alloc, node_capacity, p=p, delta=delta,
                           flags=(PX_FLAG_MEMOISE | PX_FLAG_PAIR_RESULTS) if memoise else 0, device=dev)
        pop = call.current_alloc.unsqueeze(0).repeat(P, 1, 1).contiguous()
        call.run(pop, outputs="fitness")
        for g in range(generations):      # each: the step in place, then the fitness of the children it formed
            call.generation(pop, seed, it * generations + g, max(1, P // 2), mut, outputs="fitness", inherit_rows=True)
        status = call.status()          # of the search's fitness calls, accumulated over the generations
        pollux_apply_best(call.dims, pop, call.fitness, call.current_alloc, d_best, d_K, d_nodes, d_changed)
        pollux_sim_tick(Dims(P, J, N, Gm, Gs, 0, 0), call.job_params, call.m_grid, d_K, d_nodes, d_changed, d_target,
                        interval_s, restart_delay, call.workspace, d_progress, d_goodput, d_finished)
        best = int(d_best.item())
        best_fitness = float(call.fitness[best].item())
        new_alloc = call.current_alloc.cpu().numpy()
        changed = d_changed.cpu().numpy().astype(bool)
        K = d_K.cpu().numpy()
        record = dict(interval=it, phi=job_params[PARAM_PHI].copy(), previous_alloc=state.alloc, alloc=new_alloc,
                      best_fitness=best_fitness, changed=changed, progress_before=state.progress.copy(),
                      goodput=d_goodput.cpu().numpy(), status=status, best=best)
        state.alloc = new_alloc
        state.progress = d_progress.cpu().numpy()
        state.finished = d_finished.cpu().numpy().astype(bool)
        state.interval = it + 1
        record["progress"] = state.progress.copy()
        state.history.append(dict(interval=it, best_fitness=best_fitness, gpus=int(K.sum()), changed=int(changed.sum()),
                                  finished=int(state.finished.sum())))
        if on_interval is not None:
            on_interval(state, record)
    return state
