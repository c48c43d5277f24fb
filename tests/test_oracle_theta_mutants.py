"""Do the pins of the theta_sys and loop checkers have teeth?  Each case plants one plausible mistake in a copy
of the checker's source, loads the copy as a module and asserts that a compact pin-suite rejects it, while the
unmodified source passes.  CPU only."""
import os
import types

import numpy as np
import pytest

import oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))
ORACLE_DIR = os.path.join(os.path.dirname(HERE), "oracle")

THETA_MUTANTS = [
    ("local and node pairs swapped", "np.where(nodes == 1, theta[ALPHA_SL] + theta[BETA_SL] * (K - 2),\n                           theta[ALPHA_SN] + theta[BETA_SN] * (K - 2))",
     "np.where(nodes != 1, theta[ALPHA_SL] + theta[BETA_SL] * (K - 2),\n                           theta[ALPHA_SN] + theta[BETA_SN] * (K - 2))"),
    ("sync counts from K-1", "theta[ALPHA_SL] + theta[BETA_SL] * (K - 2),", "theta[ALPHA_SL] + theta[BETA_SL] * (K - 1),"),
    ("overlap root not inverted", "np.power(np.power(tg, g) + np.power(ts, g), 1.0 / g)", "np.power(np.power(tg, g) + np.power(ts, g), g)"),
    ("accumulation counts s+1 passes", "return s * tg + last, tg, ts", "return (s + 1) * tg + last, tg, ts"),
    ("error not in logarithms", "r = np.log(pred) - np.log(np.asarray(T, np.float64))\n    return float(np.sqrt(np.mean(r * r)))",
     "r = pred - np.asarray(T, np.float64)\n    return float(np.sqrt(np.mean(r * r)))"),
    ("mean absolute instead of root mean square", "return float(np.sqrt(np.mean(r * r)))\n\n\ndef residuals", "return float(np.mean(np.abs(r)))\n\n\ndef residuals"),
    ("gradient of beta_grad without m", "J[:, BETA_G] = (s + dl_dtg) * m", "J[:, BETA_G] = (s + dl_dtg)"),
    ("gradient of the sync pair on the wrong records", "J[:, ALPHA_SL] = np.where(local, dl_dts, 0.0)", "J[:, ALPHA_SL] = np.where(node, dl_dts, 0.0)"),
    ("gamma derivative sign", "- np.log(wsum) / (g * g),", "+ np.log(wsum) / (g * g),"),
    ("prior: node pair free on one node", "    if max_nodes <= 1:\n        fixed[[ALPHA_SN, BETA_SN]] = True", "    if max_nodes <= 0:\n        fixed[[ALPHA_SN, BETA_SN]] = True"),
    ("prior: betas free with two GPUs", "    if max_k <= 2:", "    if max_k <= 1:"),
    ("gamma allowed below 1", "+ [(1.0, 10.0)]", "+ [(0.1, 10.0)]"),
    ("alphas allowed negative", "else (0.0, None) for i in range(6)]", "else (None, None) for i in range(6)]"),
]

LOOP_MUTANTS = [
    ("scale-up test not strict", "if not per_gpu[j, n] > U * ideal:", "if not per_gpu[j, n] >= U * ideal:"),
    ("scale-up compares total goodput", "out[j, n] = O.best_goodput(jb, m_grid[j], Gs, K, n)[0] / K", "out[j, n] = O.best_goodput(jb, m_grid[j], Gs, K, n)[0]"),
    ("nodes taken as GPUs", "K = n * gpus_per_node", "K = n"),
    ("growth ignores L", "while n < max_nodes and per_gpu[j, n + 1] >= L * ideal:", "while n < max_nodes and per_gpu[j, n + 1] >= 0.0 * ideal:"),
    ("growth stops one early", "while n < max_nodes and", "while n < max_nodes - 1 and"),
    ("restart delay paid by everyone", "run = dt - (restart_delay if changed[j] else 0.0)", "run = dt - restart_delay"),
    ("restart delay never paid", "run = dt - (restart_delay if changed[j] else 0.0)", "run = dt"),
    ("finished jobs keep running", "if K[j] > 0 and progress[j] < target[j]:", "if K[j] > 0:"),
    ("progress can go backwards", "            if run > 0.0:\n                new[j]", "            if True:\n                new[j]"),
]


def load_variant(filename, old=None, new=None):
    text = open(os.path.join(ORACLE_DIR, filename)).read()
    if old is not None:
        assert text.count(old) == 1, f"mutation site not found exactly once: {old!r}"
        text = text.replace(old, new)
    mod = types.ModuleType("variant_" + filename.replace(".", "_"))
    mod.__dict__["__name__"] = mod.__name__
    exec(compile(text, filename, "exec"), mod.__dict__)
    return mod


def theta_pins(TH):
    failed = []
    check = lambda name, ok: failed.append(name) if not ok else None
    theta = np.array([0.1, 0.001, 0.05, 0.01, 0.2, 0.02, 2.0])
    one = lambda K, nodes, m, s, g: TH.t_iter(np.r_[theta[:6], g], [K], [nodes], [m], [s])[0][0]
    close = lambda a, b, r=1e-10: abs(a - b) <= r * abs(b)
    check("vector 1", close(one(1, 1, 100, 0, 2.0), 0.2))
    check("vector 2", close(one(2, 1, 100, 0, 1.0), 0.25))
    check("vector 4", close(one(2, 1, 100, 1, 2.0), 0.406155281281))
    check("vector 6", close(one(4, 2, 50, 3, 3.0), 0.708127573469))
    check("vector K=3 local", close(one(3, 1, 100, 0, 1.0), 0.2 + 0.06))
    rng = np.random.default_rng(7)
    K = rng.integers(1, 17, 40)
    nodes = np.maximum(np.minimum(K, rng.integers(1, 5, 40)), 1)
    m = rng.choice([8, 32, 128], 40)
    s = rng.integers(0, 4, 40)
    T = TH.t_iter(theta, K, nodes, m, s)[0]
    check("exact fit has zero error", TH.rmsle(theta, K, nodes, m, s, T) < 1e-14)
    check("uniform factor", close(TH.rmsle(theta, K, nodes, m, s, 3.0 * T), np.log(3.0)))
    half = np.where(np.arange(40) % 2 == 0, 2.0, 1.0)
    check("half the records off", close(TH.rmsle(theta, K, nodes, m, s, T * half), np.sqrt(0.5) * np.log(2.0)))
    x = theta * 1.3
    x[6] = 3.1
    Tn = T * np.exp(0.05 * rng.standard_normal(40))
    f, g = TH.rmsle_and_gradient(x, K, nodes, m, s, Tn)
    for i in range(7):
        h = 1e-6 * max(abs(x[i]), 1e-3)
        xp, xm = x.copy(), x.copy()
        xp[i] += h
        xm[i] -= h
        num = (TH.rmsle(xp, K, nodes, m, s, Tn) - TH.rmsle(xm, K, nodes, m, s, Tn)) / (2 * h)
        check(f"gradient {i}", abs(g[i] - num) <= 1e-5 * max(abs(num), 1e-3 * np.max(np.abs(g))))
    check("prior one GPU", TH.prior_fixed([1, 1], [1, 1]).tolist() == [False, False, True, True, True, True, False])
    check("prior two GPUs", TH.prior_fixed([2, 1], [2, 1]).tolist() == [False, False, False, True, False, True, False])
    check("prior one node", TH.prior_fixed([3, 1], [1, 1]).tolist() == [False, False, False, False, True, True, False])
    # bounds: records whose best unconstrained fit wants gamma < 1 and a negative alpha_sync
    tg = 0.1 + 0.001 * m
    Tb = (s + 1) * tg + np.where(K > 1, -0.02, 0.0)                  # multi-GPU runs faster than one GPU: wants T_sync < 0
    est, _, _ = TH.fit(K, nodes, m, s, np.maximum(Tb, 0.05))
    check("alphas and betas stay non-negative", np.all(est[:6] >= 0.0) and 1.0 <= est[6] <= 10.0)
    ts = np.where(K > 1, 0.05 + 0.01 * (K - 2), 0.0)
    Tc = s * tg + np.where(K > 1, 1.6 * (tg + ts), tg)                # the last pass costs more than the sum: wants gamma < 1
    est, _, _ = TH.fit(K, nodes, m, s, Tc)
    check("gamma stays in [1, 10]", np.all(est[:6] >= 0.0) and 1.0 <= est[6] <= 10.0)
    est, err, _ = TH.fit(K, nodes, m, s, T, n_starts=3)
    check("recovery", err < 1e-8)
    return failed


def loop_pins(LP):
    failed = []
    check = lambda name, ok: failed.append(name) if not ok else None
    row = np.array([[10.0, 9.0, 8.0, 6.0, 4.9, 3.0]])
    sc = lambda now, U=2 / 3, L=0.5, t=row: int(LP.autoscale(t, [now], U, L)[0])
    check("scale 1 -> 3", sc(1) == 3)
    check("stay at 3", sc(3) == 3)
    check("strict", sc(1, U=0.9) == 1)
    check("cap", sc(1, L=0.0) == 5)
    check("L stops growth", sc(2) == 3)
    jp = np.zeros((14, 2))
    jp[0], jp[1], jp[2], jp[3], jp[4], jp[5], jp[6] = 0.1, 0.001, 0.05, 0.01, 0.2, 0.02, 2.0
    jp[7], jp[8], jp[9], jp[10], jp[11], jp[12] = 1000.0, 32.0, 4096.0, 1.0, 3600.0, 0.0
    grid = np.tile(np.array([8, 16, 32, 64], np.int32), (2, 1))
    tab = LP.goodput_per_gpu(jp, grid, 4, 4, 3)
    jb = O.job_from_params(jp, 0)
    check("ideal column", tab[0, 0] == O.best_goodput(jb, grid[0], 4, 1, 1)[0])
    check("two nodes", tab[0, 2] == O.best_goodput(jb, grid[0], 4, 8, 2)[0] / 8)
    K, nodes = np.array([2, 0], np.int32), np.array([1, 0], np.int32)
    g, new, fin = LP.sim_tick(jp, grid, 4, K, nodes, [1, 0], [10.0, 10.0], [1e9, 1e9], 60.0, 30.0)
    g0 = O.best_goodput(jb, grid[0], 4, 2, 1)[0]
    check("tick with restart", g[0] == g0 and new[0] == 10.0 + g0 * 30.0 and new[1] == 10.0)
    g, new, fin = LP.sim_tick(jp, grid, 4, K, nodes, [0, 0], [10.0, 10.0], [1e9, 1e9], 60.0, 30.0)
    check("tick without restart", new[0] == 10.0 + g0 * 60.0)
    g, new, fin = LP.sim_tick(jp, grid, 4, K, nodes, [1, 0], [10.0, 10.0], [1e9, 1e9], 20.0, 30.0)
    check("short interval", new[0] == 10.0)
    g, new, fin = LP.sim_tick(jp, grid, 4, K, nodes, [0, 0], [10.0, 10.0], [5.0, 1e9], 60.0, 30.0)
    check("finished job rests", g[0] == 0.0 and new[0] == 10.0 and fin[0])
    return failed


def test_unmodified_checkers_pass_every_pin():
    assert theta_pins(load_variant("theta.py")) == []
    assert loop_pins(load_variant("loop.py")) == []


@pytest.mark.parametrize("idx", range(len(THETA_MUTANTS)), ids=[m[0] for m in THETA_MUTANTS])
def test_a_planted_mistake_in_the_theta_checker_is_caught(idx):
    name, old, new = THETA_MUTANTS[idx]
    assert theta_pins(load_variant("theta.py", old, new)), f"no pin noticed: {name}"


@pytest.mark.parametrize("idx", range(len(LOOP_MUTANTS)), ids=[m[0] for m in LOOP_MUTANTS])
def test_a_planted_mistake_in_the_loop_checker_is_caught(idx):
    name, old, new = LOOP_MUTANTS[idx]
    assert loop_pins(load_variant("loop.py", old, new)), f"no pin noticed: {name}"
