"""ctypes binding of the CPU checker (oracle/pollux_ref.c).

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the CPU
baseline leg of the benchmark.  The GPU library never imports this package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "pollux_ref.c")
_HDR = os.path.join(_HERE, "pollux_ref.h")
_LIB = os.path.join(_HERE, "libpollux_ref.so")

NPARAM = 14
ST_BAD_PARAM, ST_ZERO_FAIR, ST_BAD_RESTART, ST_NEG_ALLOC = 1, 2, 4, 8
FLAG_NO_PENALTY, FLAG_NO_CHECK, FLAG_SAMPLE_M = 1, 2, 16


def build(force: bool = False) -> str:
    """Compile the oracle with gcc: fp64, no fused multiply-add, OpenMP over candidates."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_HDR))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-std=c11", "-O2", "-ffp-contract=off", "-fno-fast-math", "-fopenmp", "-shared", "-fPIC",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class Dims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("P", "J", "N", "Gm", "Gs", "precision", "flags")]


class Job(ctypes.Structure):
    _fields_ = [(n, ctypes.c_double) for n in
                ("alpha_g", "beta_g", "alpha_sl", "beta_sl", "alpha_sn", "beta_sn", "gamma", "phi", "M0", "Mmax", "m_mem")]


class GaParams(ctypes.Structure):
    _fields_ = [("seed", ctypes.c_uint64), ("generation", ctypes.c_uint32), ("elite_k", ctypes.c_uint32),
                ("mut_threshold", ctypes.c_uint32), ("flags", ctypes.c_uint32), ("job_gpu_cap", ctypes.c_void_p)]


_lib = None


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB)
        d, i, vp = ctypes.c_double, ctypes.c_int, ctypes.c_void_p
        L.pollux_ref_efficiency.restype = d
        L.pollux_ref_efficiency.argtypes = [d, d, d]
        L.pollux_ref_tgrad.restype = d
        L.pollux_ref_tgrad.argtypes = [d, d, d]
        L.pollux_ref_tsync.restype = d
        L.pollux_ref_tsync.argtypes = [ctypes.POINTER(Job), i, i]
        L.pollux_ref_titer.restype = d
        L.pollux_ref_titer.argtypes = [d, d, d, i]
        L.pollux_ref_goodput.restype = d
        L.pollux_ref_goodput.argtypes = [ctypes.POINTER(Job), i, i, i, i, ctypes.POINTER(ctypes.c_int)]
        L.pollux_ref_best_goodput.restype = d
        L.pollux_ref_best_goodput.argtypes = [ctypes.POINTER(Job), vp, i, i, i, i,
                                              ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
        L.pollux_ref_best_goodput_sampled.restype = d
        L.pollux_ref_best_goodput_sampled.argtypes = [ctypes.POINTER(Job), vp, i, i, i, i,
                                                      ctypes.POINTER(ctypes.c_int), ctypes.POINTER(ctypes.c_int)]
        L.pollux_ref_argmax_gap.restype = d
        L.pollux_ref_argmax_gap.argtypes = [ctypes.POINTER(Job), vp, i, i, i, i]
        L.pollux_ref_realloc_factor.restype = d
        L.pollux_ref_realloc_factor.argtypes = [d, d, d]
        L.pollux_ref_pmean.restype = d
        L.pollux_ref_pmean.argtypes = [vp, vp, i, d]
        L.pollux_ref_philox4x32_10.restype = None
        L.pollux_ref_philox4x32_10.argtypes = [vp, vp, vp]
        L.pollux_fitness_ref.restype = i
        L.pollux_fitness_ref.argtypes = [ctypes.POINTER(Dims)] + [vp] * 6 + [d, d] + [vp] * 7
        L.pollux_ga_step_ref.restype = i
        L.pollux_ga_step_ref.argtypes = [ctypes.POINTER(Dims), vp, vp, vp, ctypes.POINTER(GaParams), vp]
        L.pollux_ref_cap_row.restype = None
        L.pollux_ref_cap_row.argtypes = [vp, i, ctypes.c_int32]
        L.pollux_ref_repair.restype = None
        L.pollux_ref_repair.argtypes = [vp, i, i, vp, vp, ctypes.c_uint32, ctypes.c_uint32]
        L.pollux_ref_rank.restype = None
        L.pollux_ref_rank.argtypes = [vp, i, vp]
        L.pollux_ref_threads.restype = i
        L.pollux_ref_threads.argtypes = []
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def job(alpha_g, beta_g, alpha_sl, beta_sl, alpha_sn, beta_sn, gamma, phi, M0, Mmax, m_mem=0.0) -> Job:
    return Job(alpha_g, beta_g, alpha_sl, beta_sl, alpha_sn, beta_sn, gamma, phi, M0, Mmax, m_mem)


def job_from_params(job_params: np.ndarray, j: int) -> Job:
    return Job(*[float(job_params[k, j]) for k in range(10)], float(job_params[13, j]))


def threads() -> int:
    return lib().pollux_ref_threads()


def efficiency(phi, M0, M):
    return lib().pollux_ref_efficiency(phi, M0, M)


def tgrad(alpha_g, beta_g, m):
    return lib().pollux_ref_tgrad(alpha_g, beta_g, m)


def tsync(jb: Job, K: int, nodes: int):
    return lib().pollux_ref_tsync(ctypes.byref(jb), K, nodes)


def titer(t_grad, t_sync, gamma, s):
    return lib().pollux_ref_titer(t_grad, t_sync, gamma, s)


def goodput(jb: Job, K, nodes, m, s):
    ok = ctypes.c_int(0)
    g = lib().pollux_ref_goodput(ctypes.byref(jb), K, nodes, m, s, ctypes.byref(ok))
    return g, bool(ok.value)


def best_goodput(jb: Job, m_grid, Gs, K, nodes):
    mg = _c(m_grid, np.int32)
    im, is_ = ctypes.c_int(0), ctypes.c_int(0)
    g = lib().pollux_ref_best_goodput(ctypes.byref(jb), _p(mg), mg.size, Gs, K, nodes,
                                      ctypes.byref(im), ctypes.byref(is_))
    return g, im.value, is_.value


def best_goodput_sampled(jb: Job, M_list, s_max, K, nodes):
    """Sec. 4.3 procedure: returns (goodput, m, s)."""
    ml = _c(M_list, np.int32)
    m, s = ctypes.c_int(0), ctypes.c_int(0)
    g = lib().pollux_ref_best_goodput_sampled(ctypes.byref(jb), _p(ml), ml.size, s_max, K, nodes,
                                              ctypes.byref(m), ctypes.byref(s))
    return g, m.value, s.value


def argmax_gap(jb: Job, m_grid, Gs, K, nodes):
    mg = _c(m_grid, np.int32)
    return lib().pollux_ref_argmax_gap(ctypes.byref(jb), _p(mg), mg.size, Gs, K, nodes)


def realloc_factor(T, R, delta):
    return lib().pollux_ref_realloc_factor(T, R, delta)


def pmean(speedup, weight, p):
    s = _c(speedup, np.float64)
    w = None if weight is None else _c(weight, np.float64)
    return lib().pollux_ref_pmean(_p(s), _p(w), s.size, p)


def philox4x32_10(ctr, key):
    c = _c(ctr, np.uint32)
    k = _c(key, np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().pollux_ref_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def fitness(population, job_params, m_grid, fair_share, current_alloc, node_capacity, p, delta, Gs, flags=0):
    """Full fitness call on host arrays.  Returns a dict of outputs."""
    A = _c(population, np.int32)
    P, J, N = A.shape
    mg = _c(m_grid, np.int32)
    Gm = mg.shape[1]
    jp = _c(job_params, np.float64)
    assert jp.shape == (NPARAM, J) and mg.shape == (J, Gm)
    fs, cur, cap = _c(fair_share, np.int32), _c(current_alloc, np.int32), _c(node_capacity, np.int32)
    assert fs.shape == (J, 2) and cur.shape == (J, N) and cap.shape == (N,)
    d = Dims(P, J, N, Gm, Gs, 0, flags)
    out = dict(
        fitness=np.empty(P), best_m=np.empty((P, J), np.int32), best_s=np.empty((P, J), np.int32),
        best_goodput=np.empty((P, J)), speedup=np.empty((P, J)), violations=np.empty(P, np.int32),
    )
    st = np.zeros(1, np.int32)
    rc = lib().pollux_fitness_ref(ctypes.byref(d), _p(A), _p(jp), _p(mg), _p(fs), _p(cur), _p(cap),
                                  float(p), float(delta), _p(out["fitness"]), _p(out["best_m"]),
                                  _p(out["best_s"]), _p(out["best_goodput"]), _p(out["speedup"]),
                                  _p(out["violations"]), _p(st))
    if rc != 0:
        raise ValueError(f"pollux_fitness_ref returned {rc}")
    out["status"] = int(st[0])
    return out


GA_IN_PLACE = 1


def ga_step(parents, fitness_values, node_capacity, seed, generation, elite_k, mut_threshold, flags=0, job_gpu_cap=None):
    """One generation; with GA_IN_PLACE the result has child c in the slot of the candidate of rank c.
    job_gpu_cap: int32 [J], the most GPUs each job may hold in a child (None: no limit)."""
    A = _c(parents, np.int32)
    P, J, N = A.shape
    f = _c(fitness_values, np.float64)
    cap = _c(node_capacity, np.int32)
    d = Dims(P, J, N, 1, 1, 0, 0)
    gcap = None if job_gpu_cap is None else _c(job_gpu_cap, np.int32)
    ga = GaParams(seed, generation, elite_k, mut_threshold, flags, None if gcap is None else gcap.ctypes.data)
    out = A.copy() if flags & GA_IN_PLACE else np.empty_like(A)
    rc = lib().pollux_ga_step_ref(ctypes.byref(d), _p(out if flags & GA_IN_PLACE else A), _p(f), _p(cap), ctypes.byref(ga), _p(out))
    if rc != 0:
        raise ValueError(f"pollux_ga_step_ref returned {rc}")
    return out


def generation(population, fitness_values, job_params, m_grid, fair_share, current_alloc, node_capacity, p, delta, Gs,
               seed, generation_index, elite_k, mut_threshold, flags=0, job_gpu_cap=None):
    """One generation of the search: the step in place, then FITNESS_p of the whole new population by the plain
    definition (the library evaluates the children only; a survivor's fitness cannot have changed).
    Returns (new population, dict of fitness outputs)."""
    new = ga_step(population, fitness_values, node_capacity, seed, generation_index, elite_k, mut_threshold,
                  flags=GA_IN_PLACE, job_gpu_cap=job_gpu_cap)
    return new, fitness(new, job_params, m_grid, fair_share, current_alloc, node_capacity, p, delta, Gs, flags)


def cap_row(row, cap):
    r = np.array(row, dtype=np.int32, order="C", copy=True)
    lib().pollux_ref_cap_row(_p(r), r.size, int(cap))
    return r


def repair(A, node_capacity, seed, generation, child):
    M = np.array(A, dtype=np.int32, order="C", copy=True)
    J, N = M.shape
    cap = _c(node_capacity, np.int32)
    key = np.array([seed & 0xFFFFFFFF, seed >> 32], dtype=np.uint32)
    lib().pollux_ref_repair(_p(M), J, N, _p(cap), _p(key), generation, child)
    return M


def rank(fitness_values):
    f = _c(fitness_values, np.float64)
    order = np.empty(f.size, np.int32)
    lib().pollux_ref_rank(_p(f), f.size, _p(order))
    return order
