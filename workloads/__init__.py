"""Seeded synthetic inputs for the scheduler-search hot path.

Nothing in this package evaluates the goodput model, the fitness function or a
genetic operator: it only draws job parameters, batch-size grids, cluster
shapes and allocation matrices.  The CPU checker and the GPU library both read
the arrays produced here.

The shapes follow the cluster sizes and job mixes of the paper's evaluation
(16 nodes x 4 GPUs testbed, Sec. 5.1; larger simulated clusters, Sec. 5.3); the
parameter ranges stand in for the measured job profiles and the cluster trace,
which are not available.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libpopgen.so")
_SRC_PATH = os.path.join(_HERE, "popgen.c")

# Row order of the structure-of-arrays job parameter block [NPARAM, J].
PARAM_NAMES = (
    "alpha_grad", "beta_grad", "alpha_sync_local", "beta_sync_local",
    "alpha_sync_node", "beta_sync_node", "gamma", "phi",
    "M0", "M_max", "weight", "age_T", "restarts_R", "m_mem",
)
NPARAM = len(PARAM_NAMES)
PARAM_INDEX = {n: i for i, n in enumerate(PARAM_NAMES)}

BASE_SEED = 0x5EED2008


def build_popgen(force: bool = False) -> str:
    """Compile the allocation-matrix generator (plain C, host only)."""
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(_SRC_PATH):
        cmd = ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, _SRC_PATH, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB_PATH


_lib = None


def _popgen():
    global _lib
    if _lib is None:
        build_popgen()
        _lib = ctypes.CDLL(_LIB_PATH)
        _lib.popgen_candidates.restype = ctypes.c_int
        _lib.popgen_candidates.argtypes = [
            ctypes.c_uint64, ctypes.c_int64, ctypes.c_int64, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_int, ctypes.c_void_p,
        ]
    return _lib


@dataclass(frozen=True)
class Config:
    """One benchmark / parity configuration."""
    name: str
    index: int          # position in the list of configurations (seed offset)
    P: int              # candidates
    J: int              # jobs
    N: int              # nodes
    cap: int            # GPUs per node
    Gm: int             # points of the per-GPU batch-size grid
    Gs: int             # accumulation steps 0..Gs-1
    phi_hi: float = 1e5
    pinned_fraction: float = 0.0   # jobs whose total batch may not exceed one GPU's worth
    p: float = -1.0
    delta: float = 30.0

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index

    @property
    def evals_per_call(self) -> int:
        return self.P * self.J * self.Gm * self.Gs


CONFIGS = {
    "tiny":     Config("tiny", 0, P=16, J=8, N=4, cap=4, Gm=32, Gs=8),
    "physical": Config("physical", 1, P=100, J=30, N=16, cap=4, Gm=64, Gs=16, pinned_fraction=0.2),
    "mid":      Config("mid", 2, P=1000, J=200, N=64, cap=8, Gm=64, Gs=16, phi_hi=1e6),
    "large":    Config("large", 3, P=4096, J=1000, N=256, cap=8, Gm=128, Gs=32),
}


def fair_share(J: int, N: int, cap: int) -> np.ndarray:
    """[J,2] int32 (GPU count, nodes occupied) of an exclusive 1/J cluster share, packed."""
    kf = max(1, (N * cap) // J)
    nodes = -(-kf // cap)
    out = np.empty((J, 2), dtype=np.int32)
    out[:, 0] = kf
    out[:, 1] = nodes
    return out


def m_grid(m_max: np.ndarray, Gm: int, m_min: int = 8) -> np.ndarray:
    """[J,Gm] int32 log-spaced per-GPU batch sizes in [m_min, m_max_j] (duplicates possible)."""
    m_max = np.asarray(m_max, dtype=np.float64)
    if Gm == 1:
        return m_max.astype(np.int32).reshape(-1, 1)
    t = np.arange(Gm, dtype=np.float64) / (Gm - 1)
    g = np.floor(m_min * (m_max[:, None] / m_min) ** t[None, :] + 0.5)
    g = np.clip(g, m_min, m_max[:, None])
    return g.astype(np.int32)


def total_batch_grid(M0: np.ndarray, M_max: np.ndarray, Gm: int) -> np.ndarray:
    """[J,Gm] int32 log-spaced candidate total batch sizes in [M0_j, M_max_j] (for the sampling form of Eq. 13)."""
    M0, M_max = np.asarray(M0, np.float64), np.asarray(M_max, np.float64)
    if Gm == 1:
        return M0.astype(np.int32).reshape(-1, 1)
    t = np.arange(Gm, dtype=np.float64) / (Gm - 1)
    g = np.floor(M0[:, None] * (M_max[:, None] / M0[:, None]) ** t[None, :] + 0.5)
    return np.clip(g, M0[:, None], M_max[:, None]).astype(np.int32)


@dataclass
class Workload:
    cfg: Config
    job_params: np.ndarray      # float64 [NPARAM, J]
    m_grid: np.ndarray          # int32   [J, Gm]
    m_max: np.ndarray           # int32   [J]
    fair_share: np.ndarray      # int32   [J, 2]
    node_capacity: np.ndarray   # int32   [N]
    current_alloc: np.ndarray   # int32   [J, N]
    population: np.ndarray | None = None   # int32 [P, J, N] (None until drawn)
    extra: dict = field(default_factory=dict)

    def param(self, name: str) -> np.ndarray:
        return self.job_params[PARAM_INDEX[name]]


def draw_job_params(cfg: Config, rng: np.random.Generator) -> tuple[np.ndarray, np.ndarray]:
    """Job parameter block and per-job memory bound m_max, drawn in a fixed order."""
    J = cfg.J
    U = lambda lo, hi: rng.uniform(lo, hi, J)
    logU = lambda lo, hi: np.exp(rng.uniform(np.log(lo), np.log(hi), J))
    jp = np.zeros((NPARAM, J), dtype=np.float64)
    jp[PARAM_INDEX["alpha_grad"]] = U(0.01, 0.2)
    jp[PARAM_INDEX["beta_grad"]] = logU(1e-5, 1e-3)
    jp[PARAM_INDEX["alpha_sync_local"]] = U(0.005, 0.05)
    jp[PARAM_INDEX["beta_sync_local"]] = U(0.001, 0.01)
    jp[PARAM_INDEX["alpha_sync_node"]] = U(0.02, 0.2)
    jp[PARAM_INDEX["beta_sync_node"]] = U(0.005, 0.05)
    jp[PARAM_INDEX["gamma"]] = U(1.0, 5.0)
    jp[PARAM_INDEX["phi"]] = logU(1e2, cfg.phi_hi)
    M0 = rng.choice(np.array([32.0, 64.0, 128.0, 256.0]), J)
    m_max = rng.integers(64, 513, J).astype(np.int32)
    M_max = 32.0 * M0
    pinned = rng.uniform(0.0, 1.0, J) < cfg.pinned_fraction
    # "pinned" jobs: the total batch may not exceed what one GPU holds, but always
    # leaves one octave [M0, 2*M0] so that feasibility never hinges on divisibility
    M_max = np.where(pinned, np.maximum(2.0 * M0, m_max.astype(np.float64)), M_max)
    jp[PARAM_INDEX["M0"]] = M0
    jp[PARAM_INDEX["M_max"]] = M_max
    jp[PARAM_INDEX["weight"]] = 1.0
    age = logU(120.0, 8 * 3600.0)
    jp[PARAM_INDEX["age_T"]] = age
    jp[PARAM_INDEX["restarts_R"]] = np.floor(rng.uniform(0.0, 1.0, J) * age / 210.0)
    jp[PARAM_INDEX["m_mem"]] = m_max.astype(np.float64)      # per-GPU batch size that still fits GPU memory
    return jp, m_max


def candidates(cfg: Config, first: int, count: int, seed: int | None = None) -> np.ndarray:
    """Candidates first..first+count-1 of the configuration's population, int32 [count,J,N]."""
    kf = int(fair_share(cfg.J, cfg.N, cfg.cap)[0, 0])
    out = np.empty((count, cfg.J, cfg.N), dtype=np.int32)
    rc = _popgen().popgen_candidates(
        ctypes.c_uint64(cfg.seed if seed is None else seed), first, count, cfg.J, cfg.N, cfg.cap, kf,
        out.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise RuntimeError(f"popgen_candidates failed with {rc}")
    return out


def make(cfg: Config | str, with_population: bool = True, current: str = "random") -> Workload:
    """Draw every input of one configuration.

    current = "random": the current allocation is a separately drawn candidate
    (index P of the stream); "fair": it equals candidate 0, the packed fair share.
    """
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    rng = np.random.Generator(np.random.PCG64(cfg.seed))
    jp, m_max = draw_job_params(cfg, rng)
    cur = candidates(cfg, cfg.P if current == "random" else 0, 1)[0]
    wl = Workload(
        cfg=cfg, job_params=jp, m_grid=m_grid(m_max, cfg.Gm), m_max=m_max,
        fair_share=fair_share(cfg.J, cfg.N, cfg.cap),
        node_capacity=np.full(cfg.N, cfg.cap, dtype=np.int32),
        current_alloc=np.ascontiguousarray(cur),
    )
    if with_population:
        wl.population = candidates(cfg, 0, cfg.P)
    return wl


def sampled(wl: Workload) -> Workload:
    """The same workload for the sampling form of Eq. 13 (Sec. 4.3): the grid rows list total batch sizes."""
    import dataclasses
    return dataclasses.replace(wl, m_grid=total_batch_grid(wl.param("M0"), wl.param("M_max"), wl.cfg.Gm))


def observations(cfg: Config | str, max_obs: int = 48, seed: int | None = None) -> dict:
    """Recorded (K, nodes, m, s, T_iter) tuples per job, as a job's agent would have collected them.

    The times come from a measurement process of this module's own, not from the throughput model that is
    fitted to them: a pass costs c0 + c1 m seconds, an all-reduce a latency that grows with log2(K) and is
    dearer across nodes, the two overlap imperfectly (the longer plus 30 % of the shorter), and every
    measurement carries 3 % log-normal noise.  Jobs differ in how far they have explored: one GPU only (10 %),
    at most two GPUs (10 %), one node (30 %), several nodes (50 %).  Returns count [J] and K, nodes, m, s
    int32 [J,max_obs], T float64 [J,max_obs] (unused slots hold K = nodes = m = 1, s = 0, T = 1)."""
    if isinstance(cfg, str):
        cfg = CONFIGS[cfg]
    rng = np.random.Generator(np.random.PCG64((cfg.seed if seed is None else seed) + 0x0B5E))
    J, cap = cfg.J, cfg.cap
    _, m_max = draw_job_params(cfg, np.random.Generator(np.random.PCG64(cfg.seed)))
    grid = m_grid(m_max, 16)
    count = rng.integers(6, max_obs + 1, J).astype(np.int32)
    level = rng.choice(4, J, p=[0.1, 0.1, 0.3, 0.5])
    k_max = np.array([1, 2, cap, 4 * cap])[level]
    c0 = rng.uniform(0.01, 0.2, J)
    c1 = np.exp(rng.uniform(np.log(1e-5), np.log(1e-3), J))
    lat_local = rng.uniform(0.005, 0.05, J)
    lat_node = rng.uniform(0.02, 0.2, J)
    K = np.ones((J, max_obs), np.int32)
    nodes = np.ones((J, max_obs), np.int32)
    m = np.ones((J, max_obs), np.int32)
    s = np.zeros((J, max_obs), np.int32)
    T = np.ones((J, max_obs), np.float64)
    for j in range(J):
        n = int(count[j])
        k = rng.integers(1, k_max[j] + 1, n)
        packed = -(-k // cap)
        spread = np.minimum(k, rng.integers(1, 5, n))
        nd = np.where(rng.uniform(size=n) < 0.7, packed, np.maximum(packed, spread))
        coin = rng.uniform(size=n) < 0.5
        if level[j] == 0 or level[j] == 2:
            nd = np.ones(n, dtype=k.dtype)                       # one GPU, or one node (k <= cap)
        elif level[j] == 1:
            nd = np.where((k == 2) & coin, 2, 1)                 # two GPUs on one node or on two
        mm = grid[j, rng.integers(0, grid.shape[1], n)]
        ss = rng.integers(0, 4, n)
        compute = c0[j] + c1[j] * mm
        comm = np.where(k == 1, 0.0, np.where(nd == 1, lat_local[j], lat_node[j]) * (1.0 + 0.15 * np.log2(k)))
        t = ss * compute + np.maximum(compute, comm) + 0.3 * np.minimum(compute, comm)
        t = t * np.exp(0.03 * rng.standard_normal(n))
        K[j, :n], nodes[j, :n], m[j, :n], s[j, :n], T[j, :n] = k, nd, mm, ss, t
    return dict(count=count, K=K, nodes=nodes, m=m, s=s, T=T)


def noise_scale_schedule(phi_start: np.ndarray, growth: float = 100.0):
    """The simulated environment's gradient noise scale: it grows geometrically with training progress, from
    phi_start at the beginning to growth * phi_start at the target (the paper observes growth over training,
    Sec. 3.1; the shape here is synthetic).  Returns phi_of(fraction done) for the closed loop."""
    phi_start = np.asarray(phi_start, np.float64).copy()
    return lambda done: phi_start * growth ** np.clip(done, 0.0, 1.0)


def custom(name: str, **kw) -> Config:
    """A one-off configuration (tests use this for ragged and degenerate shapes)."""
    kw.setdefault("index", 100)
    return Config(name, **kw)
