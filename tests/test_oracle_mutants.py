"""Do the pins have teeth?  Each case plants one plausible mistake in a copy of the
CPU checker's source (a dropped term, a wrong sign or index, a swapped operand),
compiles it, and asserts that the compact pin-suite below rejects it, while the
unmodified source passes.  Everything here runs on the CPU; the mistakes never
reach the GPU.
"""
import ctypes
import os
import subprocess

import numpy as np
import pytest

import oracle as O

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "pollux_ref.c")
HDR_DIR = os.path.join(os.path.dirname(HERE), "oracle")

MUTANTS = [
    ("efficiency inverted", "return (phi + M0) / (phi + M);", "return (phi + M) / (phi + M0);"),
    ("efficiency without M0", "return (phi + M0) / (phi + M);", "return phi / (phi + M);"),
    ("T_grad drops alpha", "return alpha_g + beta_g * m;", "return beta_g * m;"),
    ("T_sync counts from K-1", "job->alpha_sl + job->beta_sl * (double)(K - 2)", "job->alpha_sl + job->beta_sl * (double)(K - 1)"),
    ("local and node pairs swapped", "if (nodes == 1) return job->alpha_sl", "if (nodes != 1) return job->alpha_sl"),
    ("overlap exponent not inverted", "1.0 / gamma);\n    return (double)s", "gamma);\n    return (double)s"),
    ("accumulation counts s+1 passes", "return (double)s * t_grad + last;", "return (double)(s + 1) * t_grad + last;"),
    ("total batch without accumulation", "double M = (double)K * (double)m * (double)(s + 1);", "double M = (double)K * (double)m;"),
    ("upper batch limit ignored", "if (M < job->M0 || M > job->Mmax) return 0.0;", "if (M < job->M0) return 0.0;"),
    ("ties go to the last index", "if (ok && g > best) { best = g; bi = i; bs = s; }", "if (ok && g >= best) { best = g; bi = i; bs = s; }"),
    ("restart factor sign", "return (age_T - restarts_R * delta) / (age_T + delta);", "return (age_T + restarts_R * delta) / (age_T + delta);"),
    ("p-mean root not inverted", "return pow(acc / wsum, 1.0 / p);", "return pow(acc / wsum, p);"),
    ("p-mean unweighted sum", "wsum += w;", "wsum += 1.0;"),
    ("speedup inverted", "double s_j = denom[j] > 0.0 ? g / denom[j] : 0.0;", "double s_j = g > 0.0 ? denom[j] / g : 0.0;"),
    ("penalty on unchanged rows", "if (use_penalty && changed && running[j])", "if (use_penalty && !changed && running[j])"),
    ("interference counts single-node jobs", "if (a > 0 && nodes_of[j] >= 2) distributed++;", "if (a > 0 && nodes_of[j] >= 1) distributed++;"),
    ("philox key not advanced", "if (round > 0) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }", "if (round > 99) { k0 += 0x9E3779B9u; k1 += 0xBB67AE85u; }"),
    ("philox words crossed", "uint32_t n0 = (uint32_t)(p1 >> 32) ^ c1 ^ k0;", "uint32_t n0 = (uint32_t)(p0 >> 32) ^ c1 ^ k0;"),
    ("rank ascending", "if (x->f > y->f) return -1;\n    if (x->f < y->f) return 1;", "if (x->f > y->f) return 1;\n    if (x->f < y->f) return -1;"),
    ("capacity repair leaves one too many", "long excess = total - cap[n];", "long excess = total - cap[n] - 1;"),
    ("sampling: s one too many", "long long s = (M + per_step - 1) / per_step - 1;", "long long s = (M + per_step - 1) / per_step;"),
    ("sampling: memory bound ignores K", "long long per_step = (long long)K * (long long)job->m_mem;", "long long per_step = (long long)job->m_mem;"),
    ("sampling: m ignores accumulation", "long long m = (M + (long long)K * (s + 1) - 1) / ((long long)K * (s + 1));", "long long m = (M + (long long)K - 1) / (long long)K;"),
    ("sampling: m rounded down", "long long m = (M + (long long)K * (s + 1) - 1) / ((long long)K * (s + 1));", "long long m = M / ((long long)K * (s + 1));"),
    ("sampling: s beyond the limit accepted", "if (s > s_max) continue;", "if (s > s_max + 100) continue;"),
    ("sampling: fair share from the dense grid", "denom[j] = sampled\n", "denom[j] = !sampled\n"),
    ("GPU limit off by one", "long room = limit - kept;", "long room = limit - kept + 1;"),
    ("GPU limit forgets what it kept", "kept += row[n];\n    }\n}", "kept += 0;\n    }\n}"),
    ("interference repair keeps the smallest holder", "if (a > most) { most = a; keep = j; }", "if (keep < 0 || a < most) { most = a; keep = j; }"),
]


def load(path):
    L = ctypes.CDLL(path)
    d, i, vp = ctypes.c_double, ctypes.c_int, ctypes.c_void_p
    L.pollux_ref_efficiency.restype = d
    L.pollux_ref_efficiency.argtypes = [d, d, d]
    L.pollux_ref_tgrad.restype = d
    L.pollux_ref_tgrad.argtypes = [d, d, d]
    L.pollux_ref_tsync.restype = d
    L.pollux_ref_tsync.argtypes = [ctypes.POINTER(O.Job), i, i]
    L.pollux_ref_titer.restype = d
    L.pollux_ref_titer.argtypes = [d, d, d, i]
    L.pollux_ref_goodput.restype = d
    L.pollux_ref_goodput.argtypes = [ctypes.POINTER(O.Job), i, i, i, i, ctypes.POINTER(ctypes.c_int)]
    L.pollux_ref_best_goodput.restype = d
    L.pollux_ref_best_goodput.argtypes = [ctypes.POINTER(O.Job), vp, i, i, i, i, ctypes.POINTER(ctypes.c_int),
                                          ctypes.POINTER(ctypes.c_int)]
    L.pollux_ref_best_goodput_sampled.restype = d
    L.pollux_ref_best_goodput_sampled.argtypes = [ctypes.POINTER(O.Job), vp, i, i, i, i, ctypes.POINTER(ctypes.c_int),
                                                  ctypes.POINTER(ctypes.c_int)]
    L.pollux_ref_realloc_factor.restype = d
    L.pollux_ref_realloc_factor.argtypes = [d, d, d]
    L.pollux_ref_pmean.restype = d
    L.pollux_ref_pmean.argtypes = [vp, vp, i, d]
    L.pollux_ref_philox4x32_10.restype = None
    L.pollux_ref_philox4x32_10.argtypes = [vp, vp, vp]
    L.pollux_fitness_ref.restype = i
    L.pollux_fitness_ref.argtypes = [ctypes.POINTER(O.Dims)] + [vp] * 6 + [d, d] + [vp] * 7
    L.pollux_ref_cap_row.restype = None
    L.pollux_ref_cap_row.argtypes = [vp, i, ctypes.c_int32]
    L.pollux_ref_repair.restype = None
    L.pollux_ref_repair.argtypes = [vp, i, i, vp, vp, ctypes.c_uint32, ctypes.c_uint32]
    L.pollux_ref_rank.restype = None
    L.pollux_ref_rank.argtypes = [vp, i, vp]
    return L


def ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def pin_suite(L):
    """A compact version of the pins in test_oracle_*.py; returns the list of failed pins."""
    failed = []

    def check(name, ok):
        if not ok:
            failed.append(name)

    close = lambda a, b, r=1e-9: abs(a - b) <= r * abs(b)
    jb2 = O.job(0.1, 0.001, 0.05, 0.01, 0.2, 0.02, 2.0, 1000.0, 100.0, 3200.0)
    jb3 = O.job(0.1, 0.001, 0.05, 0.01, 0.2, 0.02, 3.0, 1000.0, 100.0, 3200.0)
    ok = ctypes.c_int(0)
    gp = lambda jb, K, n, m, s: L.pollux_ref_goodput(ctypes.byref(jb), K, n, m, s, ctypes.byref(ok))
    # closed forms
    check("efficiency is 1 at M0", L.pollux_ref_efficiency(1000.0, 100.0, 100.0) == 1.0)
    check("efficiency 11/12", close(L.pollux_ref_efficiency(1000.0, 100.0, 200.0), 11.0 / 12.0))
    check("tgrad", L.pollux_ref_tgrad(0.1, 0.001, 100.0) == 0.1 + 0.001 * 100.0)
    check("tsync K=1", L.pollux_ref_tsync(ctypes.byref(jb2), 1, 1) == 0.0)
    check("tsync local", L.pollux_ref_tsync(ctypes.byref(jb2), 2, 1) == 0.05 and close(L.pollux_ref_tsync(ctypes.byref(jb2), 3, 1), 0.06))
    check("tsync node", L.pollux_ref_tsync(ctypes.byref(jb2), 2, 2) == 0.2 and close(L.pollux_ref_tsync(ctypes.byref(jb2), 4, 2), 0.24))
    check("overlap 3-4-5", close(L.pollux_ref_titer(0.3, 0.4, 2.0, 0), 0.5, 1e-14))
    check("overlap gamma=1", L.pollux_ref_titer(0.2, 0.05, 1.0, 0) == 0.25)
    check("accumulation", close(L.pollux_ref_titer(0.15, 0.24, 3.0, 4) - L.pollux_ref_titer(0.15, 0.24, 3.0, 0), 0.6, 1e-12))
    # hand-derived vectors (tests/golden/goodput_vectors.txt)
    check("vector 1", close(gp(jb2, 1, 1, 100, 0), 500.0))
    check("vector 3", close(gp(jb2, 2, 1, 100, 0), 889.2972918))
    check("vector 4", close(gp(jb2, 2, 1, 100, 1), 773.806789597))
    check("vector 5", close(gp(jb2, 4, 2, 100, 0), 1006.00405662))
    check("vector 6", close(gp(jb3, 4, 2, 50, 3), 690.396627961))
    check("M above the limit is infeasible", gp(jb2, 4, 1, 100, 8) == 0.0 and ok.value == 0)
    # argmax ties
    grid = np.array([100, 100, 100], dtype=np.int32)
    im, is_ = ctypes.c_int(0), ctypes.c_int(0)
    L.pollux_ref_best_goodput(ctypes.byref(jb2), ptr(grid), 3, 4, 1, 1, ctypes.byref(im), ctypes.byref(is_))
    check("ties to the lowest index", (im.value, is_.value) == (0, 0))
    # Sec. 4.3 sampling, points worked out by hand for K = 2 GPUs and a memory bound of 64 per GPU:
    #   M = 128 -> one pass holds it: s = 0, m = 64;  M = 129 -> s = 1, m = ceil(129/4) = 33;
    #   M = 300 -> 128 per pass: s = 2, m = ceil(300/6) = 50;  M = 1000 -> s = 7, m = 63
    jm = O.job(0.1, 0.001, 0.05, 0.01, 0.2, 0.02, 2.0, 1000.0, 100.0, 3200.0, 64.0)

    def sampled(Ms, s_max, K=2, nodes=1):
        arr = np.array(Ms, dtype=np.int32)
        L.pollux_ref_best_goodput_sampled(ctypes.byref(jm), ptr(arr), len(Ms), s_max, K, nodes, ctypes.byref(im), ctypes.byref(is_))
        return im.value, is_.value

    check("sampling M=128", sampled([128], 15) == (64, 0))
    check("sampling M=129", sampled([129], 15) == (33, 1))
    check("sampling M=300", sampled([300], 15) == (50, 2))
    check("sampling M=1000", sampled([1000], 15) == (63, 7))
    check("sampling s limit", sampled([1000], 3) == (-1, -1))
    check("sampling one GPU", sampled([300], 15, K=1) == (60, 4))
    arr = np.array([128, 129, 300, 1000], dtype=np.int32)
    gs = L.pollux_ref_best_goodput_sampled(ctypes.byref(jm), ptr(arr), 4, 15, 2, 1, ctypes.byref(im), ctypes.byref(is_))
    pts = [(64, 0), (33, 1), (50, 2), (63, 7)]
    vals = [gp(jm, 2, 1, m, s) for m, s in pts]
    check("sampling takes the best point", gs == max(vals) and (im.value, is_.value) == pts[int(np.argmax(vals))])
    # restart factor, p-mean
    check("restart factor", close(L.pollux_ref_realloc_factor(3600.0, 2.0, 30.0), 3540.0 / 3630.0))
    S = np.array([1.0, 2.0, 0.5, 4.0])
    check("harmonic mean", close(L.pollux_ref_pmean(ptr(S), None, 4, -1.0), 16.0 / 15.0))
    check("p = -10", close(L.pollux_ref_pmean(ptr(S), None, 4, -10.0), 0.574293064048))
    w = np.array([3.0, 1.0])
    S2 = np.array([1.0, 4.0])
    check("weights", close(L.pollux_ref_pmean(ptr(S2), ptr(w), 2, 1.0), 1.75))
    # Philox known answer
    out = np.zeros(4, np.uint32)
    c = np.array([0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344], np.uint32)
    k = np.array([0xa4093822, 0x299f31d0], np.uint32)
    L.pollux_ref_philox4x32_10(ptr(c), ptr(k), ptr(out))
    check("philox", list(out) == [0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1])
    # rank
    f = np.array([0.5, 0.7, 0.5, -1.0])
    order = np.zeros(4, np.int32)
    L.pollux_ref_rank(ptr(f), 4, ptr(order))
    check("rank", list(order) == [1, 0, 2, 3])
    # repair
    cap = np.array([4], np.int32)
    A = np.array([[3], [2], [0], [4]], np.int32)
    key = np.array([1, 2], np.uint32)
    L.pollux_ref_repair(ptr(A), 4, 1, ptr(cap), ptr(key), 0, 0)
    check("capacity repair", int(A.sum()) == 4)
    cap3 = np.full(3, 8, np.int32)
    B = np.array([[1, 2, 0], [0, 3, 1], [0, 2, 0]], np.int32)
    L.pollux_ref_repair(ptr(B), 3, 3, ptr(cap3), ptr(key), 0, 0)
    check("interference repair", B.tolist() == [[1, 0, 0], [0, 3, 1], [0, 2, 0]])
    # per-job GPU limit: kept in ascending node order
    row = np.array([3, 0, 2, 4], np.int32)
    L.pollux_ref_cap_row(ptr(row), 4, 4)
    check("GPU limit 4 on (3,0,2,4)", row.tolist() == [3, 0, 1, 0])
    row = np.array([3, 0, 2, 4], np.int32)
    L.pollux_ref_cap_row(ptr(row), 4, 9)
    check("GPU limit not reached", row.tolist() == [3, 0, 2, 4])
    # whole call: the fair-share candidate scores exactly 1; a changed row is penalised; violations
    J, N, Gm, Gs = 3, 3, 8, 3
    jp = np.zeros((14, J))
    jp[0], jp[1], jp[2], jp[3], jp[4], jp[5] = 0.1, 0.001, 0.05, 0.01, 0.2, 0.02
    jp[6], jp[7], jp[8], jp[9], jp[10], jp[11], jp[12] = 2.0, 1000.0, 32.0, 1024.0, [1.0, 2.0, 1.0], 3600.0, 2.0
    mg = np.tile(np.array([8, 16, 32, 64, 96, 128, 192, 256], np.int32), (J, 1))
    fs = np.tile(np.array([2, 1], np.int32), (J, 1))
    cur = np.array([[2, 0, 0], [0, 2, 0], [0, 0, 2]], np.int32)
    pop = np.stack([cur, np.array([[2, 0, 0], [0, 1, 0], [0, 0, 2]], np.int32),
                    np.array([[2, 2, 0], [0, 1, 1], [3, 0, 0]], np.int32)])
    capn = np.full(N, 4, np.int32)
    d = O.Dims(3, J, N, Gm, Gs, 0, 0)
    fit = np.zeros(3)
    bm, bs = np.zeros((3, J), np.int32), np.zeros((3, J), np.int32)
    bg, sp = np.zeros((3, J)), np.zeros((3, J))
    viol, st = np.zeros(3, np.int32), np.zeros(1, np.int32)
    L.pollux_fitness_ref(ctypes.byref(d), ptr(pop), ptr(jp), ptr(mg), ptr(fs), ptr(cur), ptr(capn), -1.0, 30.0,
                         ptr(fit), ptr(bm), ptr(bs), ptr(bg), ptr(sp), ptr(viol), ptr(st))
    check("fair share scores 1", fit[0] == 1.0 and np.all(sp[0] == 1.0))
    check("unchanged rows are not penalised", sp[1, 0] == 1.0 and sp[1, 2] == 1.0)
    check("changed row is penalised", sp[1, 1] < bg[1, 1] / bg[0, 1] and close(sp[1, 1], bg[1, 1] / bg[0, 1] * 3540.0 / 3630.0))
    check("fewer GPUs, lower goodput", bg[1, 1] < bg[0, 1])
    check("violations", list(viol) == [0, 0, 2] and fit[2] == -2.0)
    S1 = sp[1]
    check("weighted harmonic mean in the call", close(fit[1], 4.0 / (1.0 / S1[0] + 2.0 / S1[1] + 1.0 / S1[2]), 1e-12))
    # the same call with the sampling argmax: the grid row now lists total batch sizes; memory bound 40 per GPU
    jp[13] = 40.0
    Ml = np.tile(np.array([32, 64, 100, 160, 256, 400, 640, 1024], np.int32), (J, 1))
    d16 = O.Dims(3, J, N, Gm, Gs, 0, 16)
    L.pollux_fitness_ref(ctypes.byref(d16), ptr(pop), ptr(jp), ptr(Ml), ptr(fs), ptr(cur), ptr(capn), -1.0, 30.0,
                         ptr(fit), ptr(bm), ptr(bs), ptr(bg), ptr(sp), ptr(viol), ptr(st))
    # two GPUs, at most 3 passes of 80: M = 160 -> (40, 1); 256 -> s = 3 is beyond Gs-1 = 2; 100 -> (25, 1); 64 -> (32, 0)
    jq = O.job(0.1, 0.001, 0.05, 0.01, 0.2, 0.02, 2.0, 1000.0, 32.0, 1024.0, 40.0)
    cand = [(16, 0), (32, 0), (25, 1), (40, 1)]
    vals = [gp(jq, 2, 1, m, s) for m, s in cand]
    check("sampled call: fair share scores 1", fit[0] == 1.0 and np.all(sp[0] == 1.0))
    check("sampled call: chosen point", (int(bm[0, 0]), int(bs[0, 0])) == cand[int(np.argmax(vals))] and bg[0, 0] == max(vals))
    return failed


@pytest.fixture(scope="module")
def workdir(tmp_path_factory):
    return tmp_path_factory.mktemp("mutants")


def build_variant(workdir, name, text):
    src = os.path.join(str(workdir), name + ".c")
    so = os.path.join(str(workdir), name + ".so")
    with open(src, "w") as f:
        f.write(text)
    subprocess.run(["gcc", "-std=c11", "-O1", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-I", HDR_DIR, "-o", so,
                    src, "-lm"], check=True)
    return load(so)


def test_the_unmodified_oracle_passes_every_pin(workdir):
    assert pin_suite(build_variant(workdir, "original", open(SRC).read())) == []


@pytest.mark.parametrize("idx", range(len(MUTANTS)), ids=[m[0] for m in MUTANTS])
def test_a_planted_mistake_is_caught(workdir, idx):
    name, old, new = MUTANTS[idx]
    text = open(SRC).read()
    assert text.count(old) == 1, f"mutation site for '{name}' not found exactly once"
    failed = pin_suite(build_variant(workdir, f"mutant{idx}", text.replace(old, new)))
    assert failed, f"no pin noticed: {name}"
