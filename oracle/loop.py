"""CPU checker for the two consumers of the goodput argmax outside the search itself
(Pollux, arXiv 2008.12260): the goodput-based auto-scaling rule (Sec. 5.3.3, "Cloud
auto-scaling") and one tick of a discrete-time simulation of the jobs (Sec. 5.3,
"Simulator construction" / "Simulator fidelity").

TEST INFRASTRUCTURE ONLY.  Plain Python loops over jobs; every goodput value comes from the
argmax of Eq. 13 in oracle/pollux_ref.c (best_goodput).

Readings
  * Auto-scaling.  The rule is stated for one job that holds whole nodes: with a = n nodes of c GPUs each,
    scale up when  max GOODPUT(a) / SUM(a)  >  U * max GOODPUT(one GPU),  to a node count at which the predicted
    goodput per GPU is "approximately" L of that ideal.  Here: starting from the current count, nodes are added
    one at a time while the next count still predicts at least L of the ideal per GPU (and max_nodes is not
    exceeded); a job that does not meet the U condition keeps its count.  n nodes are taken as K = n c GPUs on
    n nodes (one node: the local synchronisation pair, Eq. 9).
  * Simulator tick.  The paper replays measured profiles; what is kept is its bookkeeping: over an interval
    of dt seconds a job advances by goodput x (dt - restart delay), the delay (30 s in the paper) being paid
    by a job whose allocation was changed in this interval; a job with no GPUs does not advance; a job is
    finished when its progress reaches its target.  The goodput is the maximum of Eq. 13 at the job's current
    (K, nodes), i.e. with the batch size and accumulation steps its agent would choose.
  * Applying the search's outcome (Sec. 4.3: the allocation matrix with the highest fitness is applied).  The
    best candidate is the first in the search's ranking (fitness descending, lowest index among equals, NaN
    last); a job is re-allocated when its row changes and it held GPUs before (Sec. 4.2).
"""
from __future__ import annotations

import numpy as np

import oracle as O


def goodput_per_gpu(job_params, m_grid, Gs, gpus_per_node, max_nodes):
    """[J, max_nodes + 1]: column 0 = best goodput on one GPU (the ideal per GPU under perfect scaling);
    column n >= 1 = best goodput on n full nodes divided by the GPUs held."""
    J = m_grid.shape[0]
    out = np.zeros((J, max_nodes + 1))
    for j in range(J):
        jb = O.job_from_params(job_params, j)
        out[j, 0] = O.best_goodput(jb, m_grid[j], Gs, 1, 1)[0]
        for n in range(1, max_nodes + 1):
            K = n * gpus_per_node
            out[j, n] = O.best_goodput(jb, m_grid[j], Gs, K, n)[0] / K
    return out


def autoscale(per_gpu, nodes_now, U, L):
    """Sec. 5.3.3 on a table from goodput_per_gpu(): the new node count of every job."""
    J, cols = per_gpu.shape
    max_nodes = cols - 1
    new = np.array(nodes_now, dtype=np.int32).copy()
    for j in range(J):
        n = int(new[j])
        if n < 1 or n > max_nodes:
            continue
        ideal = per_gpu[j, 0]
        if not per_gpu[j, n] > U * ideal:
            continue
        while n < max_nodes and per_gpu[j, n + 1] >= L * ideal:
            n += 1
        new[j] = n
    return new


def sim_tick(job_params, m_grid, Gs, K, nodes, changed, progress, target, dt, restart_delay):
    """One interval of the discrete-time simulation.  Returns (goodput [J], new progress [J], finished [J])."""
    J = m_grid.shape[0]
    goodput = np.zeros(J)
    new = np.array(progress, dtype=np.float64).copy()
    for j in range(J):
        if K[j] > 0 and progress[j] < target[j]:
            goodput[j] = O.best_goodput(O.job_from_params(job_params, j), m_grid[j], Gs, int(K[j]), int(nodes[j]))[0]
            run = dt - (restart_delay if changed[j] else 0.0)
            if run > 0.0:
                new[j] = progress[j] + goodput[j] * run
    return goodput, new, new >= np.asarray(target, np.float64)


def apply_best(population, fitness, current_alloc):
    """The end of a scheduling interval: (index of the best candidate, its matrix, K [J], nodes [J], changed [J])."""
    f = np.asarray(fitness, np.float64)
    best, best_f = -1, -np.inf
    for c in range(len(f)):
        v = f[c] if f[c] == f[c] else -np.inf
        if best < 0 or v > best_f:
            best, best_f = c, v
    new = np.array(population[best], dtype=np.int32, copy=True)
    cur = np.asarray(current_alloc)
    K = new.sum(axis=1).astype(np.int32)
    nodes = (new > 0).sum(axis=1).astype(np.int32)
    changed = (new != cur).any(axis=1) & (cur.sum(axis=1) > 0)
    return best, new, K, nodes, changed
