"""Thin Python binding of libpollux_hip.so (C ABI in include/pollux.h).

Argument marshalling only: every step of the path runs in the HIP kernels.
torch is used for device memory and streams.  There is no CPU fallback: if the
library has not been built, importing the entry points raises.
"""
from __future__ import annotations

import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libpollux_hip.so")

NPARAM = 14
PARAM_PHI = 7            # row of job_params that holds the gradient noise scale (PX_PHI)
PX_OK, PX_E_INVALID_ARG, PX_E_WORKSPACE, PX_E_UNSUPPORTED_ARCH, PX_E_HIP = 0, -1, -2, -3, -4
PX_FLAG_NO_REALLOC_PENALTY, PX_FLAG_NO_CONSTRAINT_CHECK, PX_FLAG_MEMOISE, PX_FLAG_KEEP_JOB_TABLES = 1, 2, 4, 8
PX_FLAG_SAMPLE_M = 16
PX_FLAG_PAIR_RESULTS = 32
PX_GA_IN_PLACE = 1
PX_GA_INHERIT_ROWS = 2
PX_ST_BAD_PARAM, PX_ST_ZERO_FAIR, PX_ST_BAD_RESTART, PX_ST_NEG_ALLOC = 1, 2, 4, 8

EXPORTS = ("pollux_version", "pollux_strerror", "pollux_workspace_size", "pollux_fitness", "pollux_fitness_static",
           "pollux_ga_step",
           "pollux_fit_theta", "pollux_goodput_per_gpu", "pollux_autoscale", "pollux_sim_tick", "pollux_last_status",
           "pollux_fitness_timed", "pollux_apply_best", "pollux_generation")


class PolluxError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


class Dims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("P", "J", "N", "Gm", "Gs", "precision", "flags")]


class GaParams(ctypes.Structure):
    _fields_ = [("seed", ctypes.c_uint64), ("generation", ctypes.c_uint32), ("elite_k", ctypes.c_uint32),
                ("mut_threshold", ctypes.c_uint32), ("flags", ctypes.c_uint32), ("job_gpu_cap", ctypes.c_void_p)]


_lib = None


def lib() -> ctypes.CDLL:
    """Load the built library; raise if it is missing (no fallback of any kind)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        vp, i, d, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_double, ctypes.c_size_t
        L.pollux_version.restype = i
        L.pollux_version.argtypes = []
        L.pollux_strerror.restype = ctypes.c_char_p
        L.pollux_strerror.argtypes = [i]
        L.pollux_workspace_size.restype = i
        L.pollux_workspace_size.argtypes = [ctypes.POINTER(Dims), ctypes.POINTER(sz)]
        L.pollux_fitness.restype = i
        L.pollux_fitness.argtypes = [ctypes.POINTER(Dims)] + [vp] * 6 + [d, d, vp, sz] + [vp] * 6 + [vp]
        L.pollux_fitness_static.restype = i
        L.pollux_fitness_static.argtypes = [ctypes.POINTER(Dims)] + [vp] * 6 + [d, d] + [vp] * 7 + [vp]
        L.pollux_ga_step.restype = i
        L.pollux_ga_step.argtypes = [ctypes.POINTER(Dims), vp, vp, vp, ctypes.POINTER(GaParams), vp, sz, vp, vp]
        L.pollux_fit_theta.restype = i
        L.pollux_fit_theta.argtypes = [ctypes.c_int32, ctypes.c_int32] + [vp] * 7 + [ctypes.c_int32, ctypes.c_int32] + [vp] * 4
        L.pollux_goodput_per_gpu.restype = i
        L.pollux_goodput_per_gpu.argtypes = [ctypes.POINTER(Dims), vp, vp, ctypes.c_int32, ctypes.c_int32, vp, sz, vp, vp]
        L.pollux_autoscale.restype = i
        L.pollux_autoscale.argtypes = [ctypes.c_int32, ctypes.c_int32, vp, vp, d, d, vp, vp]
        L.pollux_sim_tick.restype = i
        L.pollux_sim_tick.argtypes = [ctypes.POINTER(Dims)] + [vp] * 6 + [d, d, vp, sz, vp, vp, vp, vp]
        L.pollux_last_status.restype = i
        L.pollux_last_status.argtypes = [vp, vp, ctypes.POINTER(ctypes.c_int32)]
        L.pollux_fitness_timed.restype = i
        L.pollux_fitness_timed.argtypes = [ctypes.POINTER(Dims)] + [vp] * 6 + [d, d, vp, sz] + [vp] * 6 + [vp, vp, vp]
        L.pollux_generation.restype = i
        L.pollux_generation.argtypes = ([ctypes.POINTER(Dims)] + [vp] * 6 + [d, d, ctypes.POINTER(GaParams), vp, sz]
                                        + [vp] * 6 + [vp])
        L.pollux_apply_best.restype = i
        L.pollux_apply_best.argtypes = [ctypes.POINTER(Dims)] + [vp] * 7 + [vp]
        _lib = L
    return _lib


def version() -> int:
    return lib().pollux_version()


def strerror(code: int) -> str:
    return lib().pollux_strerror(code).decode()


def workspace_size(dims: Dims) -> int:
    n = ctypes.c_size_t(0)
    rc = lib().pollux_workspace_size(ctypes.byref(dims), ctypes.byref(n))
    if rc != PX_OK:
        raise PolluxError(rc, "pollux_workspace_size")
    return n.value


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream_handle(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def pollux_fitness(dims: Dims, population, job_params, m_grid, fair_share, current_alloc, node_capacity,
                   p: float, delta: float, workspace, fitness, best_m, best_s, best_goodput=None, speedup=None,
                   violations=None, stream=None, sweep_events=None) -> None:
    """pollux_fitness of the C ABI on torch device tensors (already allocated, contiguous); with
    sweep_events = (start, stop), two torch.cuda.Event objects, pollux_fitness_timed."""
    args = [ctypes.byref(dims), _ptr(population), _ptr(job_params), _ptr(m_grid), _ptr(fair_share), _ptr(current_alloc),
            _ptr(node_capacity), float(p), float(delta), _ptr(workspace), workspace.numel() * workspace.element_size(),
            _ptr(fitness), _ptr(best_m), _ptr(best_s), _ptr(best_goodput), _ptr(speedup), _ptr(violations)]
    if sweep_events is None:
        rc = lib().pollux_fitness(*args, _stream_handle(stream))
    else:
        rc = lib().pollux_fitness_timed(*args, ctypes.c_void_p(sweep_events[0].cuda_event),
                                        ctypes.c_void_p(sweep_events[1].cuda_event), _stream_handle(stream))
    if rc != PX_OK:
        raise PolluxError(rc, "pollux_fitness")


STATIC_SCRATCH_BYTES = 64 << 20


def pollux_fitness_static(dims: Dims, population, job_params, m_grid, fair_share, current_alloc, node_capacity,
                          p: float, delta: float, fitness, best_m, best_s, best_goodput=None, speedup=None,
                          violations=None, status=None, stream=None) -> None:
    """pollux_fitness_static of the C ABI: no workspace argument, the library's own scratch array is used."""
    rc = lib().pollux_fitness_static(
        ctypes.byref(dims), _ptr(population), _ptr(job_params), _ptr(m_grid), _ptr(fair_share), _ptr(current_alloc),
        _ptr(node_capacity), float(p), float(delta), _ptr(fitness), _ptr(best_m), _ptr(best_s), _ptr(best_goodput),
        _ptr(speedup), _ptr(violations), _ptr(status), _stream_handle(stream))
    if rc != PX_OK:
        raise PolluxError(rc, "pollux_fitness_static")


def pollux_ga_step(dims: Dims, parents, fitness, node_capacity, ga: GaParams, workspace, children, stream=None) -> None:
    """pollux_ga_step of the C ABI on torch device tensors."""
    rc = lib().pollux_ga_step(
        ctypes.byref(dims), _ptr(parents), _ptr(fitness), _ptr(node_capacity), ctypes.byref(ga), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _ptr(children), _stream_handle(stream))
    if rc != PX_OK:
        raise PolluxError(rc, "pollux_ga_step")


def pollux_fit_theta(obs_count, obs_K, obs_nodes, obs_m, obs_s, obs_T, theta, rmsle, iterations=None, theta_init=None,
                     max_iter=200, n_starts=3, stream=None) -> None:
    """pollux_fit_theta of the C ABI on torch device tensors (records [J,max_obs], outputs theta [7,J], rmsle [J])."""
    J, max_obs = obs_K.shape
    rc = lib().pollux_fit_theta(J, max_obs, _ptr(obs_count), _ptr(obs_K), _ptr(obs_nodes), _ptr(obs_m), _ptr(obs_s),
                                _ptr(obs_T), _ptr(theta_init), max_iter, n_starts, _ptr(theta), _ptr(rmsle), _ptr(iterations),
                                _stream_handle(stream))
    if rc != PX_OK:
        raise PolluxError(rc, "pollux_fit_theta")


def fit_theta(records: dict, theta_init=None, max_iter=200, n_starts=3, device="cuda", stream=None) -> dict:
    """Marshal host record arrays (count [J]; K, nodes, m, s int32 [J,max_obs]; T float64 [J,max_obs]) to the
    device, call pollux_fit_theta and return theta [7,J], rmsle [J], iterations [J] as numpy arrays."""
    import numpy as np
    import torch
    dev = torch.device(device)
    i32 = lambda a: torch.as_tensor(np.ascontiguousarray(a, dtype=np.int32)).to(dev)
    count, K, nodes, m, s = (i32(records[k]) for k in ("count", "K", "nodes", "m", "s"))
    T = torch.as_tensor(np.ascontiguousarray(records["T"], dtype=np.float64)).to(dev)
    J = K.shape[0]
    theta = torch.empty((7, J), dtype=torch.float64, device=dev)
    rmsle = torch.empty(J, dtype=torch.float64, device=dev)
    iters = torch.empty(J, dtype=torch.int32, device=dev)
    init = None if theta_init is None else torch.as_tensor(np.ascontiguousarray(theta_init, dtype=np.float64)).to(dev)
    pollux_fit_theta(count, K, nodes, m, s, T, theta, rmsle, iters, init, max_iter, n_starts, stream)
    torch.cuda.synchronize()
    return dict(theta=theta.cpu().numpy(), rmsle=rmsle.cpu().numpy(), iterations=iters.cpu().numpy())


def pollux_goodput_per_gpu(dims: Dims, job_params, m_grid, gpus_per_node, max_nodes, workspace, per_gpu, stream=None) -> None:
    rc = lib().pollux_goodput_per_gpu(ctypes.byref(dims), _ptr(job_params), _ptr(m_grid), gpus_per_node, max_nodes,
                                      _ptr(workspace), workspace.numel() * workspace.element_size(), _ptr(per_gpu),
                                      _stream_handle(stream))
    if rc != PX_OK:
        raise PolluxError(rc, "pollux_goodput_per_gpu")


def pollux_autoscale(per_gpu, nodes_now, U, L, nodes_new, stream=None) -> None:
    J, cols = per_gpu.shape
    rc = lib().pollux_autoscale(J, cols - 1, _ptr(per_gpu), _ptr(nodes_now), U, L, _ptr(nodes_new), _stream_handle(stream))
    if rc != PX_OK:
        raise PolluxError(rc, "pollux_autoscale")


def pollux_sim_tick(dims: Dims, job_params, m_grid, K, nodes, changed, target, dt, restart_delay, workspace, progress,
                    goodput, finished, stream=None) -> None:
    rc = lib().pollux_sim_tick(ctypes.byref(dims), _ptr(job_params), _ptr(m_grid), _ptr(K), _ptr(nodes), _ptr(changed),
                               _ptr(target), dt, restart_delay, _ptr(workspace),
                               workspace.numel() * workspace.element_size(), _ptr(progress), _ptr(goodput),
                               _ptr(finished), _stream_handle(stream))
    if rc != PX_OK:
        raise PolluxError(rc, "pollux_sim_tick")


def pollux_last_status(workspace, stream=None) -> int:
    out = ctypes.c_int32(0)
    rc = lib().pollux_last_status(_ptr(workspace), _stream_handle(stream), ctypes.byref(out))
    if rc != PX_OK:
        raise PolluxError(rc, "pollux_last_status")
    return out.value


def pollux_generation(dims: Dims, population, job_params, m_grid, fair_share, current_alloc, node_capacity, p: float,
                      delta: float, ga: GaParams, workspace, fitness, best_m, best_s, best_goodput=None, speedup=None,
                      violations=None, stream=None) -> None:
    """pollux_generation of the C ABI on torch device tensors: the search step in place, then the fitness of its children."""
    rc = lib().pollux_generation(
        ctypes.byref(dims), _ptr(population), _ptr(job_params), _ptr(m_grid), _ptr(fair_share), _ptr(current_alloc),
        _ptr(node_capacity), float(p), float(delta), ctypes.byref(ga), _ptr(workspace),
        workspace.numel() * workspace.element_size(), _ptr(fitness), _ptr(best_m), _ptr(best_s), _ptr(best_goodput),
        _ptr(speedup), _ptr(violations), _stream_handle(stream))
    if rc != PX_OK:
        raise PolluxError(rc, "pollux_generation")


def pollux_apply_best(dims: Dims, population, fitness, current_alloc, best, K, nodes, changed, stream=None) -> None:
    """pollux_apply_best of the C ABI on torch device tensors (current_alloc is overwritten)."""
    rc = lib().pollux_apply_best(ctypes.byref(dims), _ptr(population), _ptr(fitness), _ptr(current_alloc), _ptr(best),
                                 _ptr(K), _ptr(nodes), _ptr(changed), _stream_handle(stream))
    if rc != PX_OK:
        raise PolluxError(rc, "pollux_apply_best")


class FitnessCall:
    """Device buffers of one configuration plus the two entry points bound to them.

    Allocation happens here, once; `run()` and `ga_step()` only marshal pointers.
    """

    def __init__(self, P, J, N, Gm, Gs, job_params, m_grid, fair_share, current_alloc, node_capacity,
                 p=-1.0, delta=30.0, flags=0, precision=0, device="cuda:0"):
        import torch
        self.torch = torch
        self.dims = Dims(P, J, N, Gm, Gs, precision, flags)
        self.p, self.delta = float(p), float(delta)
        dev = torch.device(device)
        as_dev = lambda a, dt: torch.as_tensor(a, dtype=dt).contiguous().to(dev)
        self.job_params = as_dev(job_params, torch.float64)
        self.m_grid = as_dev(m_grid, torch.int32)
        self.fair_share = as_dev(fair_share, torch.int32)
        self.current_alloc = as_dev(current_alloc, torch.int32)
        self.node_capacity = as_dev(node_capacity, torch.int32)
        assert self.job_params.shape == (NPARAM, J) and self.m_grid.shape == (J, Gm)
        assert self.fair_share.shape == (J, 2) and self.current_alloc.shape == (J, N) and self.node_capacity.shape == (N,)
        self.workspace = torch.empty(workspace_size(self.dims), dtype=torch.uint8, device=dev)
        assert self.workspace.data_ptr() % 256 == 0
        if os.environ.get("POLLUX_POISON_WORKSPACE"):
            # for tests: nothing in the library may depend on what a fresh workspace holds (0xFF bytes read as NaN / -1)
            self.workspace.fill_(0xFF)
        self.fitness = torch.empty(P, dtype=torch.float64, device=dev)
        self.best_m = torch.empty((P, J), dtype=torch.int32, device=dev)
        self.best_s = torch.empty((P, J), dtype=torch.int32, device=dev)
        self.best_goodput = torch.empty((P, J), dtype=torch.float64, device=dev)
        self.speedup = torch.empty((P, J), dtype=torch.float64, device=dev)
        self.violations = torch.empty(P, dtype=torch.int32, device=dev)

    def run(self, population, stream=None, outputs="all", keep_job_tables=False, sweep_events=None):
        """outputs: "all"; "argmax" (fitness, violations, best_m, best_s); "fitness" (fitness and violations only)."""
        assert outputs in ("all", "argmax", "fitness")
        full, argmax = outputs == "all", outputs != "fitness"
        dims = self.dims
        if keep_job_tables:
            dims = Dims(dims.P, dims.J, dims.N, dims.Gm, dims.Gs, dims.precision, dims.flags | PX_FLAG_KEEP_JOB_TABLES)
        pollux_fitness(dims, population, self.job_params, self.m_grid, self.fair_share, self.current_alloc,
                       self.node_capacity, self.p, self.delta, self.workspace, self.fitness,
                       self.best_m if argmax else None, self.best_s if argmax else None,
                       self.best_goodput if full else None, self.speedup if full else None, self.violations,
                       stream, sweep_events)

    def status(self, stream=None) -> int:
        return pollux_last_status(self.workspace, stream)

    def ga_step(self, parents, children, seed, generation, elite_k, mut_threshold, fitness=None, stream=None,
                flags=0, job_gpu_cap=None):
        """job_gpu_cap: int32 device tensor [J] (the most GPUs each job may hold in a child) or None."""
        if job_gpu_cap is not None:
            assert job_gpu_cap.dtype == self.torch.int32 and job_gpu_cap.numel() == self.dims.J and job_gpu_cap.is_cuda
        ga = GaParams(seed, generation, elite_k, mut_threshold, flags, None if job_gpu_cap is None else job_gpu_cap.data_ptr())
        pollux_ga_step(self.dims, parents, self.fitness if fitness is None else fitness, self.node_capacity, ga,
                       self.workspace, children, stream)

    def generation(self, population, seed, generation, elite_k, mut_threshold, stream=None, outputs="all", job_gpu_cap=None,
                   inherit_rows=False):
        """pollux_generation on this call's buffers: search step in place, then the fitness of the children only.
        inherit_rows: PX_GA_INHERIT_ROWS (rows a child holds unchanged take over their parent's results)."""
        assert outputs in ("all", "argmax", "fitness")
        full, argmax = outputs == "all", outputs != "fitness"
        ga = GaParams(seed, generation, elite_k, mut_threshold, PX_GA_IN_PLACE | (PX_GA_INHERIT_ROWS if inherit_rows else 0),
                      None if job_gpu_cap is None else job_gpu_cap.data_ptr())
        pollux_generation(self.dims, population, self.job_params, self.m_grid, self.fair_share, self.current_alloc,
                          self.node_capacity, self.p, self.delta, ga, self.workspace, self.fitness,
                          self.best_m if argmax else None, self.best_s if argmax else None,
                          self.best_goodput if full else None, self.speedup if full else None, self.violations, stream)

    def results(self) -> dict:
        self.torch.cuda.synchronize()
        return dict(fitness=self.fitness.cpu().numpy(), best_m=self.best_m.cpu().numpy(),
                    best_s=self.best_s.cpu().numpy(), best_goodput=self.best_goodput.cpu().numpy(),
                    speedup=self.speedup.cpu().numpy(), violations=self.violations.cpu().numpy(),
                    status=self.status())
