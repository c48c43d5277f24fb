"""GPU checks of pollux_fit_theta against the CPU checker (oracle/theta.py).

The fit is a local minimisation of a function with several local minima, run by two different algorithms (the
library: damped Gauss-Newton; the checker: scipy's L-BFGS-B, the routine the paper names), so the end points
are compared as follows:
  * the error the library reports equals the checker's error function at the library's parameters (1e-12);
  * bounds and exploration priors hold exactly;
  * the library's end point is a minimum for the checker too: L-BFGS-B started there gains less than 1e-6;
  * started from the checker's end point, the library never ends worse, and typically ends at the same error;
  * over a workload, the library's error is within 0.1 % of the best of the checker's seven starts (a start
    policy of its own, see oracle/theta.py), or lower, for at least 97 % of jobs;
  * records generated from known parameters are reproduced to rounding, every job.
"""
import numpy as np
import pytest

import oracle.theta as TH
import workloads as W

pytestmark = pytest.mark.gpu


def job_records(ob, j):
    n = ob["count"][j]
    return tuple(ob[k][j, :n] for k in ("K", "nodes", "m", "s", "T"))


def pack(recs, max_obs):
    J = len(recs)
    out = dict(count=np.zeros(J, np.int32), K=np.ones((J, max_obs), np.int32), nodes=np.ones((J, max_obs), np.int32),
               m=np.ones((J, max_obs), np.int32), s=np.zeros((J, max_obs), np.int32), T=np.ones((J, max_obs)))
    for j, (K, nodes, m, s, T) in enumerate(recs):
        n = len(K)
        out["count"][j] = n
        out["K"][j, :n], out["nodes"][j, :n], out["m"][j, :n], out["s"][j, :n], out["T"][j, :n] = K, nodes, m, s, T
    return out


def exact_records(rng, n, max_k, theta):
    K = rng.integers(1, max_k + 1, n)
    nodes = np.maximum(np.where(rng.uniform(size=n) < 0.7, -(-K // 4), np.minimum(K, rng.integers(1, 5, n))), 1)
    m = rng.choice([8, 16, 32, 64, 128, 256], n)
    s = rng.integers(0, 4, n)
    return K, nodes, m, s, TH.t_iter(theta, K, nodes, m, s)[0]


@pytest.mark.parametrize("name", ["physical", "mid"])
def test_fit_on_generated_records(name):
    import paper_2008_12260_amd as px
    ob = W.observations(name)
    J = ob["K"].shape[0]
    got = px.fit_theta(ob, max_iter=300, n_starts=3)
    theta, err = got["theta"], got["rmsle"]
    assert np.all(theta[:6] >= 0.0) and np.all(theta[6] >= 1.0) and np.all(theta[6] <= 10.0)
    close = 0
    for j in range(J):
        r = job_records(ob, j)
        # the reported error is the checker's error function at the reported parameters (a job with fewer records
        # than parameters is fitted exactly: both errors are then rounding noise around 1e-16)
        assert abs(TH.rmsle(theta[:, j], *r) - err[j]) <= 1e-12 * err[j] + 1e-14
        # priors
        assert np.all(theta[TH.prior_fixed(r[0], r[1]), j] == 0.0)
        want = TH.fit(*r, n_starts=7)[1]
        close += err[j] <= want * 1.001 + 1e-12
    print(f"{name}: {close} of {J} fits within 0.1 % of the checker's best or lower")
    assert close >= 0.97 * J, f"only {close} of {J} fits are as good as the checker's"


def test_end_points_are_minima_for_the_checker_too():
    import paper_2008_12260_amd as px
    ob = W.observations("physical")
    got = px.fit_theta(ob, max_iter=300, n_starts=3)
    for j in range(ob["K"].shape[0]):
        r = job_records(ob, j)
        polished = TH.fit(*r, start=got["theta"][:, j])[1]
        assert polished >= got["rmsle"][j] * (1.0 - 1e-6), (j, polished, got["rmsle"][j])


def test_started_from_the_checkers_end_point_the_library_stays_there():
    import paper_2008_12260_amd as px
    ob = W.observations("physical")
    J = ob["K"].shape[0]
    init = np.zeros((7, J))
    want = np.zeros(J)
    for j in range(J):
        init[:, j], want[j], _ = TH.fit(*job_records(ob, j), n_starts=3)
    got = px.fit_theta(ob, theta_init=init, max_iter=300, n_starts=1)
    assert np.all(got["rmsle"] <= want * (1 + 1e-12))                      # never worse than where it started
    assert np.median(got["rmsle"] / want) > 1 - 1e-6                       # and, typically, no better: the same minimum


def test_exact_records_are_reproduced():
    import paper_2008_12260_amd as px
    rng = np.random.default_rng(21)
    base = np.array([0.1, 0.001, 0.05, 0.01, 0.2, 0.02, 2.0])
    recs, truth = [], []
    for _ in range(40):
        th = base * np.exp(0.4 * rng.standard_normal(7))
        th[6] = rng.uniform(1.2, 6.0)
        truth.append(th)
        recs.append(exact_records(rng, int(rng.integers(20, 100)), 16, th))
    ob = pack(recs, 128)                                                    # more than one record per lane
    got = px.fit_theta(ob, max_iter=300, n_starts=3)
    good = got["rmsle"] < 1e-9
    assert good.all(), got["rmsle"]
    for j in np.flatnonzero(good):
        K, nodes, m, s, T = recs[j]
        assert np.max(np.abs(TH.t_iter(got["theta"][:, j], K, nodes, m, s)[0] / T - 1.0)) < 1e-7


def test_priors_degenerate_inputs_and_argument_checks():
    import torch
    import paper_2008_12260_amd as px
    rng = np.random.default_rng(22)
    base = np.array([0.1, 0.001, 0.05, 0.01, 0.2, 0.02, 2.0])
    one_gpu = exact_records(rng, 12, 1, base)
    two_gpus = exact_records(rng, 12, 2, base)
    one_node = list(exact_records(rng, 30, 4, base))
    one_node[1] = np.ones_like(one_node[1])
    one_node[4] = TH.t_iter(base, *one_node[:4])[0]
    single = exact_records(rng, 1, 16, base)
    empty = tuple(np.zeros(0, x.dtype) for x in single)
    ob = pack([one_gpu, two_gpus, tuple(one_node), single, empty], 32)
    got = px.fit_theta(ob, max_iter=300, n_starts=3)
    th = got["theta"]
    assert np.all(th[2:6, 0] == 0.0) and got["rmsle"][0] < 1e-9
    assert th[3, 1] == 0.0 and th[5, 1] == 0.0
    assert th[4, 2] == 0.0 and th[5, 2] == 0.0 and th[2, 2] > 0.0
    assert np.isfinite(th[:, 3]).all() and got["rmsle"][3] < 1e-9          # one record: fitted exactly
    assert th[:, 4].tolist() == [0, 0, 0, 0, 0, 0, 1] and got["rmsle"][4] == 0.0 and got["iterations"][4] == 0
    # determinism
    again = px.fit_theta(ob, max_iter=300, n_starts=3)
    assert np.array_equal(again["theta"], th) and np.array_equal(again["rmsle"], got["rmsle"])
    # argument checks
    z = torch.zeros((2, 4), dtype=torch.int32, device="cuda")
    t = torch.ones((2, 4), dtype=torch.float64, device="cuda")
    out, e = torch.zeros((7, 2), dtype=torch.float64, device="cuda"), torch.zeros(2, dtype=torch.float64, device="cuda")
    with pytest.raises(px.PolluxError):
        px.pollux_fit_theta(z[:, 0].contiguous(), z, z, z, z, t, out, e, n_starts=0)
    with pytest.raises(px.PolluxError):
        px.pollux_fit_theta(z[:, 0].contiguous(), z, z, z, z, t, out, e, n_starts=6)
    with pytest.raises(px.PolluxError):
        px.pollux_fit_theta(z[:, 0].contiguous(), z, z, z, z, t, out, e, max_iter=-1)


def test_bounds_bind_where_the_unconstrained_fit_would_leave_the_box():
    """Records that want T_sync < 0 (several GPUs faster than the model allows) and records that want gamma < 1
    (a last pass dearer than T_grad + T_sync): the fit must end on the bound, and match the checker's error."""
    import paper_2008_12260_amd as px
    rng = np.random.default_rng(23)
    K = rng.integers(1, 17, 40)
    nodes = np.maximum(np.minimum(K, rng.integers(1, 5, 40)), 1)
    m = rng.choice([8, 32, 128], 40)
    s = rng.integers(0, 4, 40)
    tg = 0.1 + 0.001 * m
    fast = np.maximum((s + 1) * tg + np.where(K > 1, -0.02, 0.0), 0.05)
    ts = np.where(K > 1, 0.05 + 0.01 * (K - 2), 0.0)
    dear = s * tg + np.where(K > 1, 1.6 * (tg + ts), tg)
    ob = pack([(K, nodes, m, s, fast), (K, nodes, m, s, dear)], 64)
    got = px.fit_theta(ob, max_iter=300, n_starts=5)       # the best corner of the first job is reached from the fifth start only
    th = got["theta"]
    assert np.all(th[:6] >= 0.0) and np.all(th[6] >= 1.0) and np.all(th[6] <= 10.0)
    assert th[6, 1] == 1.0                                              # gamma pressed against its lower bound
    for j, T in enumerate((fast, dear)):
        assert abs(TH.rmsle(th[:, j], K, nodes, m, s, T) - got["rmsle"][j]) <= 1e-12 * got["rmsle"][j]
        want = TH.fit(K, nodes, m, s, T, n_starts=3)[1]
        assert got["rmsle"][j] <= want * 1.001
