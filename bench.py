#!/usr/bin/env python3
"""Benchmark of the PolluxSched search hot path on one MI355X.

A step is one generation on the large configuration (4096 candidates, 1000
jobs, 256 nodes x 8 GPUs, 128 x 32 grid): pollux_fitness on the current
population followed by pollux_ga_step in place (children overwrite the candidates
that did not survive).  The reported
value counts the (m, s) grid points the fitness call sweeps
(P * J * Gm * Gs per step) over the wall time of the whole step.

Prints one JSON line.  Inputs are synthetic and resident in HBM before the
timed region starts.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP64_VECTOR_PEAK_TFLOPS = 78.6      # 256 CUs x 4 SIMDs x 16 lanes x 2 (FMA) x 2.4 GHz
FLOPS_PER_EVAL = 7                  # Eq. 4 at one grid point: 5 add/mul + 2 divisions, each counted as one
# Counter figures of the sweep kernel on the "large" workload, from rocprofv3 runs of this file (summaries and commands
# under profiles/).  They describe the kernel they were taken on: `source_sha256` is the digest of the library's
# sources at that time (kernel_source_digest()), and the bench line reports them only while the digest still matches;
# after any change to the sources they are reported as null until the counters are taken again.
#   traffic_bytes   HBM bytes per launch: FETCH_SIZE and WRITE_SIZE, each scaled by what the same counter reads for a
#                   device-to-device copy of known size in the same run
#   fp64_flops      64 lanes x (ADD_F64 + MUL_F64 + 2 x FMA_F64 wave-instructions) per launch
#   valu_insts      vector instructions per launch; scan_insts = those of the scan itself (2.25 per grid point)
#   valu_busy       fraction of the kernel's cycles in which the vector ALUs were busy
PROFILED = {
    "large": {
        "source_sha256": "9fc9005fe7fdea90975db54cb86c8be87596f71b8f68e43c9cc4102ab6256aad",
        "traffic_bytes": 2_079_137 * 1024 * 2 + 698_183 * 1024,      # FETCH_SIZE x 2.0 + WRITE_SIZE x 1.0 (launches that store m*, s*)
        "fp64_flops": 64 * (8.960e5 + 1.770e7 + 2 * 2.670e8),
        "valu_insts": 9.95523e8,
        "scan_insts": 2.25 * 1.6777e10 / 64,
        "valu_busy": 1.01368e9 * 4 / 1024 / (3.37224e7 / 8),           # SQ_ACTIVE_INST_VALU x 4 cycles / SIMDs / cycles
    },
}
GA_SEED = 0x2008_1226_5EED_0001
def mut_threshold(J):               # mutation probability 1/J per job: about one move per child
    return (1 << 32) // J


def kernel_source_digest():
    """sha256 over the library's sources and its build script (what the compiled kernels are a function of)."""
    import hashlib
    h = hashlib.sha256()
    base = os.path.join(ROOT, "paper_2008_12260_amd")
    files = sorted(os.path.join("csrc", f) for f in os.listdir(os.path.join(base, "csrc"))) + ["build.py"]
    for f in files + [os.path.join("..", "include", "pollux.h")]:
        h.update(f.encode())
        h.update(open(os.path.join(base, f), "rb").read())
    return h.hexdigest()


def host_description():
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    return {"cpu_model": model, "nproc": os.cpu_count(), "affinity_cpus": len(os.sched_getaffinity(0))}


def compiler_version():
    """The compiler that built the library, as the build wrote it down beside the library (no child process here:
    a process that holds the GPU should not start one)."""
    try:
        with open(os.path.join(ROOT, "paper_2008_12260_amd", "libpollux_hip.so.buildinfo")) as f:
            return f.read().strip()
    except OSError:
        return None


def cpu_baseline(wl, cfg, target_seconds=30.0):
    """The CPU checker, as it stands, on a bounded sample of the same workload (fitness + search step)."""
    import numpy as np
    import oracle as O
    import workloads as W

    def one(count):
        pop = W.candidates(cfg, 0, count)
        t0 = time.perf_counter()
        r = O.fitness(pop, wl.job_params, wl.m_grid, wl.fair_share, wl.current_alloc, wl.node_capacity,
                      cfg.p, cfg.delta, cfg.Gs)
        O.ga_step(pop, r["fitness"], wl.node_capacity, GA_SEED, 0, max(1, count // 2), mut_threshold(cfg.J),
                  flags=O.GA_IN_PLACE)
        return time.perf_counter() - t0

    probe = 32
    t_probe = one(probe)
    count = int(min(cfg.P, max(64, probe * target_seconds / max(t_probe, 1e-6))))
    count = max(64, (count // 64) * 64)
    t = one(count)
    evals = count * cfg.J * cfg.Gm * cfg.Gs
    return {
        "value": evals / t, "unit": "evals/s", "cores": O.threads(), "kind": "oracle",
        "sample": f"candidates 0..{count - 1} of {cfg.P} (all {cfg.J} jobs, full {cfg.Gm}x{cfg.Gs} grid), "
                  f"fitness + one search step, {t:.2f} s",
        "seconds": t, **host_description(),
        "full_population_seconds_extrapolated": t * cfg.P / count,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="large", choices=["large", "mid", "physical", "tiny"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ga-loop", action="store_true")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="after the timed region, copy the population device-to-device twice (a plain copy of known "
                         "size against which HBM byte counters are scaled)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU; a population would shard over candidates, "
                 "but no multi-GPU path exists. Use --gpus 1.")

    import numpy as np
    import torch
    import paper_2008_12260_amd as px
    import workloads as W

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    dev = torch.device("cuda:0")
    cfg = W.CONFIGS[args.workload]
    wl = W.make(cfg, with_population=False)
    host_pop = W.candidates(cfg, 0, cfg.P)
    call = px.FitnessCall(cfg.P, cfg.J, cfg.N, cfg.Gm, cfg.Gs, wl.job_params, wl.m_grid, wl.fair_share,
                          wl.current_alloc, wl.node_capacity, p=cfg.p, delta=cfg.delta, device=dev)
    a = torch.from_numpy(host_pop).to(dev)
    del host_pop
    stream = torch.cuda.current_stream()
    elite = cfg.P // 2

    gen = 0
    for _ in range(args.warmup):
        call.run(a, stream=stream, outputs="argmax")
        call.ga_step(a, a, GA_SEED, gen, elite, mut_threshold(cfg.J), stream=stream, flags=px.PX_GA_IN_PLACE)
        gen += 1
    torch.cuda.synchronize()

    # timed region: exactly --steps generations; the sweep kernel of every step is bracketed by its own events
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    fit_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    for e0, e1 in ev + fit_ev:          # create the underlying HIP events before the clock starts
        e0.record(stream); e1.record(stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        fit_ev[k][0].record(stream)
        call.run(a, stream=stream, outputs="argmax", sweep_events=ev[k])       # full call every step: job-level kernels included; (m*, s*) of every pair written
        fit_ev[k][1].record(stream)
        call.ga_step(a, a, GA_SEED, gen, elite, mut_threshold(cfg.J), stream=stream, flags=px.PX_GA_IN_PLACE)
        gen += 1
    torch.cuda.synchronize()
    t1 = time.perf_counter()

    # The next generations with pollux_generation, twice from the same population and with the same generation
    # numbers (so both loops form the same matrices): the step in place and then (i) the fitness of the 2048
    # children only (a survivor's results cannot change within a scheduling interval; only the children's grid
    # points are counted), (ii) with PX_GA_INHERIT_ROWS, of the children only the rows a move or a repair has
    # changed are read back and swept, an unchanged row takes over its parent's results.  How many rows the repairs
    # touch depends on how far the search has converged (two-parent children of unlike parents need many).
    b = a.clone()
    gen_loop = gen
    loop_s, loop_best = {}, {}
    for inherit in (False, True):
        if inherit:
            a.copy_(b)
        g = gen_loop
        call.run(a, stream=stream, outputs="fitness")
        for _ in range(2):
            call.generation(a, GA_SEED, g, elite, mut_threshold(cfg.J), stream=stream, outputs="fitness", inherit_rows=inherit)
            g += 1
        torch.cuda.synchronize()
        ti0 = time.perf_counter()
        for _ in range(args.steps):
            call.generation(a, GA_SEED, g, elite, mut_threshold(cfg.J), stream=stream, outputs="fitness", inherit_rows=inherit)
            g += 1
        torch.cuda.synchronize()
        loop_s[inherit] = time.perf_counter() - ti0
        loop_best[inherit] = float(call.fitness.max().item())
    gen = g
    incremental_s, inherited_s = loop_s[False], loop_s[True]

    # the same search step out of place (survivors copied into a second buffer), for comparison
    o0, o1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    call.ga_step(a, b, GA_SEED, gen, elite, mut_threshold(cfg.J), stream=stream)
    o0.record(stream)
    for k in range(3):
        call.ga_step(a, b, GA_SEED, gen + k, elite, mut_threshold(cfg.J), stream=stream)
    o1.record(stream)
    torch.cuda.synchronize()
    ga_out_of_place_ms = o0.elapsed_time(o1) / 3

    if args.calibration_copy:
        for _ in range(2):
            b.copy_(a)
        torch.cuda.synchronize()
    del b

    status = call.status()
    best_fitness = float(call.fitness.max().item())
    elapsed = t1 - t0
    evals_per_step = cfg.evals_per_call
    sweep_ms = [e0.elapsed_time(e1) for e0, e1 in ev]
    fit_ms = [e0.elapsed_time(e1) for e0, e1 in fit_ev]
    sweep_avg_ms = sum(sweep_ms) / len(sweep_ms)
    achieved_tflops = evals_per_step * FLOPS_PER_EVAL / (sweep_avg_ms * 1e-3) / 1e12

    extra = {
        "fitness_call_ms": sum(fit_ms) / len(fit_ms),
        "sweep_kernel_ms": sweep_avg_ms,
        "ga_step_ms": elapsed * 1e3 / args.steps - sum(fit_ms) / len(fit_ms),
        "ga_step_out_of_place_ms": ga_out_of_place_ms,
        "fitness_only_evals_per_s": evals_per_step / (sum(fit_ms) / len(fit_ms) * 1e-3),
        "sweep_kernel_evals_per_s": evals_per_step / (sweep_avg_ms * 1e-3),
        "population_bytes_per_s_in_sweep": 4.0 * cfg.P * cfg.J * cfg.N / (sweep_avg_ms * 1e-3),
        "status_word": status, "best_fitness_after_run": best_fitness, "seed": cfg.seed,
        "children_only_generations_per_s": args.steps / incremental_s,
        "children_only_ms_per_generation": incremental_s * 1e3 / args.steps,
        "children_only_evals_per_s": (cfg.P - elite) * cfg.J * cfg.Gm * cfg.Gs * args.steps / incremental_s,
        "children_only_best_fitness": loop_best[False], "changed_rows_only_best_fitness": loop_best[True],
        "changed_rows_only_generations_per_s": args.steps / inherited_s,
        "changed_rows_only_ms_per_generation": inherited_s * 1e3 / args.steps,
    }

    # memoised mode (one sweep per (job, K, placement class); not part of the headline: its population pass
    # looks results up instead of sweeping, so its grid points are not counted)
    mcall_memo = px.FitnessCall(cfg.P, cfg.J, cfg.N, cfg.Gm, cfg.Gs, wl.job_params, wl.m_grid, wl.fair_share,
                                wl.current_alloc, wl.node_capacity, p=cfg.p, delta=cfg.delta,
                                flags=px.PX_FLAG_MEMOISE, device=dev)
    # timed with (m*, s*) of every pair written ("argmax") and with fitness and violations only, which is all a search
    # needs ("fitness_only": 33 MB of stores less per call)
    for mode, key in (("argmax", "memoised_fitness_call_ms"), ("fitness", "memoised_fitness_only_call_ms")):
        for _ in range(2):
            mcall_memo.run(a, stream=stream, outputs=mode)
        m0, m1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        m0.record(stream)
        for _ in range(5):
            mcall_memo.run(a, stream=stream, outputs=mode)
        m1.record(stream)
        torch.cuda.synchronize()
        extra[key] = m0.elapsed_time(m1) / 5
    extra["memoised_population_bytes_per_s"] = 4.0 * cfg.P * cfg.J * cfg.N / (extra["memoised_fitness_call_ms"] * 1e-3)
    del mcall_memo

    # the argmax by sampling total batch sizes (Sec. 4.3): Gm evaluations of Eq. 4 per pair instead of Gm x Gs; its
    # own figure, not part of the headline (the grid row of a job then lists total batch sizes)
    swl = W.sampled(wl)
    scall = px.FitnessCall(cfg.P, cfg.J, cfg.N, cfg.Gm, cfg.Gs, swl.job_params, swl.m_grid, swl.fair_share,
                           swl.current_alloc, swl.node_capacity, p=cfg.p, delta=cfg.delta,
                           flags=px.PX_FLAG_SAMPLE_M, device=dev)
    for _ in range(2):
        scall.run(a, stream=stream)
    s0, s1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    s0.record(stream)
    for _ in range(5):
        scall.run(a, stream=stream)
    s1.record(stream)
    torch.cuda.synchronize()
    extra["sampled_fitness_call_ms"] = s0.elapsed_time(s1) / 5
    extra["sampled_evals_per_s"] = cfg.P * cfg.J * cfg.Gm / (extra["sampled_fitness_call_ms"] * 1e-3)
    del scall, swl

    if not args.no_ga_loop:
        # the search loop on the mid configuration: 100 generations, fitness + step each; job tables are kept
        # between generations (the jobs do not change within a scheduling interval).  Timed twice: with the
        # full sweep per (candidate, job), and in memoised mode (identical matrices and fitness).
        mcfg = W.CONFIGS["mid"]
        mwl = W.make(mcfg)
        for label, flags, mut in (("ga_loop_mid", 0, mut_threshold(mcfg.J)),
                                  ("ga_loop_mid_memoised", px.PX_FLAG_MEMOISE | px.PX_FLAG_PAIR_RESULTS, mut_threshold(mcfg.J)),
                                  ("ga_loop_mid_mutation_1_in_8", 0, 1 << 29)):
            mcall = px.FitnessCall(mcfg.P, mcfg.J, mcfg.N, mcfg.Gm, mcfg.Gs, mwl.job_params, mwl.m_grid,
                                   mwl.fair_share, mwl.current_alloc, mwl.node_capacity, p=mcfg.p, delta=mcfg.delta,
                                   flags=flags, device=dev)
            ma = torch.from_numpy(mwl.population).to(dev)
            for g in range(5):
                mcall.run(ma, stream=stream, outputs="fitness")
                mcall.ga_step(ma, ma, GA_SEED, g, mcfg.P // 2, mut, stream=stream, flags=px.PX_GA_IN_PLACE)
            torch.cuda.synchronize()
            tg0 = time.perf_counter()
            for g in range(5, 105):
                mcall.run(ma, stream=stream, outputs="fitness", keep_job_tables=True)
                mcall.ga_step(ma, ma, GA_SEED, g, mcfg.P // 2, mut, stream=stream, flags=px.PX_GA_IN_PLACE)
            torch.cuda.synchronize()
            tg1 = time.perf_counter()
            extra[label + "_generations_per_s"] = 100.0 / (tg1 - tg0)
            if not flags:
                extra[label + "_evals_per_s"] = 100.0 * mcfg.evals_per_call / (tg1 - tg0)
            extra[label + "_best_fitness"] = float(mcall.fitness.max().item())
            # the same loop with pollux_generation (children only)
            ma = torch.from_numpy(mwl.population).to(dev)
            mcall.run(ma, stream=stream, outputs="fitness")
            for g in range(5):
                mcall.generation(ma, GA_SEED, g, mcfg.P // 2, mut, stream=stream, outputs="fitness")
            torch.cuda.synchronize()
            tg0 = time.perf_counter()
            for g in range(5, 105):
                mcall.generation(ma, GA_SEED, g, mcfg.P // 2, mut, stream=stream, outputs="fitness")
            torch.cuda.synchronize()
            extra[label + "_children_only_generations_per_s"] = 100.0 / (time.perf_counter() - tg0)
            extra[label + "_children_only_best_fitness"] = float(mcall.fitness.max().item())
            # and with PX_GA_INHERIT_ROWS (only the rows a move or a repair has changed are swept)
            ma = torch.from_numpy(mwl.population).to(dev)
            mcall.run(ma, stream=stream, outputs="fitness")
            for g in range(5):
                mcall.generation(ma, GA_SEED, g, mcfg.P // 2, mut, stream=stream, outputs="fitness", inherit_rows=True)
            torch.cuda.synchronize()
            tg0 = time.perf_counter()
            for g in range(5, 105):
                mcall.generation(ma, GA_SEED, g, mcfg.P // 2, mut, stream=stream, outputs="fitness", inherit_rows=True)
            torch.cuda.synchronize()
            extra[label + "_changed_rows_only_generations_per_s"] = 100.0 / (time.perf_counter() - tg0)
            extra[label + "_changed_rows_only_best_fitness"] = float(mcall.fitness.max().item())

        # one fitness call on the mid configuration at three values of the fairness knob, in fp64 and in fp32
        # arithmetic (launch overhead included: five to six small kernels per call)
        ma = torch.from_numpy(mwl.population).to(dev)
        matrix = {}
        for pname, precision in (("fp64", 0), ("fp32", 1)):
            for knob in (-1.0, 0.5, 1.0):
                mcall = px.FitnessCall(mcfg.P, mcfg.J, mcfg.N, mcfg.Gm, mcfg.Gs, mwl.job_params, mwl.m_grid,
                                       mwl.fair_share, mwl.current_alloc, mwl.node_capacity, p=knob, delta=mcfg.delta,
                                       precision=precision, device=dev)
                for _ in range(3):
                    mcall.run(ma, stream=stream, outputs="fitness")
                f0, f1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                f0.record(stream)
                for _ in range(20):
                    mcall.run(ma, stream=stream, outputs="fitness")
                f1.record(stream)
                torch.cuda.synchronize()
                matrix[f"{pname}_p={knob:g}"] = f0.elapsed_time(f1) / 20
        extra["mid_fitness_call_ms"] = matrix
        extra["mid_fitness_call_fp64_ms"] = matrix["fp64_p=-1"]
        extra["mid_fitness_call_fp32_ms"] = matrix["fp32_p=-1"]
        extra["mid_fitness_call_evals_per_s"] = {k: mcfg.evals_per_call / (v * 1e-3) for k, v in matrix.items()}

    # the step before the path: theta_sys of all jobs of the workload fitted to synthetic records (Sec. 4.1)
    records = W.observations(cfg, max_obs=48)
    i32 = lambda x: torch.as_tensor(np.ascontiguousarray(x, dtype=np.int32)).to(dev)
    rec_dev = [i32(records[k]) for k in ("count", "K", "nodes", "m", "s")] + [torch.as_tensor(records["T"]).to(dev)]
    th_out = torch.empty((7, cfg.J), dtype=torch.float64, device=dev)
    err_out = torch.empty(cfg.J, dtype=torch.float64, device=dev)
    px.pollux_fit_theta(*rec_dev, th_out, err_out, max_iter=300, n_starts=3, stream=stream)
    q0, q1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    q0.record(stream)
    for _ in range(3):
        px.pollux_fit_theta(*rec_dev, th_out, err_out, max_iter=300, n_starts=3, stream=stream)
    q1.record(stream)
    torch.cuda.synchronize()
    extra["theta_fit_ms"] = q0.elapsed_time(q1) / 3
    extra["theta_fit_jobs"] = cfg.J
    extra["theta_fit_median_rmsle"] = float(err_out.median().item())

    if not args.no_ga_loop:
        # the scheduling loop on the mid configuration: per interval 20 generations from the current allocation,
        # the best matrix applied, one simulator tick (the paper reports about 1 s per 60 s interval on one vCPU)
        from paper_2008_12260_amd import closed_loop
        lwl = W.make("mid", with_population=False, current="fair")
        lcfg = lwl.cfg
        largs = (lwl.job_params, lwl.m_grid, lwl.fair_share, lwl.node_capacity, np.full(lcfg.J, 1e7),
                 W.noise_scale_schedule(lwl.param("phi")), lwl.current_alloc)
        lkw = dict(P=lcfg.P, Gs=lcfg.Gs, p=lcfg.p, delta=lcfg.delta, generations=20, seed=GA_SEED)
        closed_loop.run(*largs, intervals=1, **lkw)
        tl0 = time.perf_counter()
        lstate = closed_loop.run(*largs, intervals=5, **lkw)
        extra["closed_loop_mid_ms_per_interval"] = (time.perf_counter() - tl0) * 1e3 / 5
        extra["closed_loop_mid_best_fitness"] = lstate.history[-1]["best_fitness"]

    prof = PROFILED.get(cfg.name)
    if prof is not None and prof.get("source_sha256") != kernel_source_digest():
        prof = None                  # the kernels have changed since the counters were taken
    roofline = {
        "bound": "alu", "achieved": achieved_tflops, "peak": FP64_VECTOR_PEAK_TFLOPS, "unit": "TFLOP/s",
        "frac": achieved_tflops / FP64_VECTOR_PEAK_TFLOPS, "traffic": prof["traffic_bytes"] if prof else None,
        "kernel": "px::pairs_kernel", "flops_per_eval": FLOPS_PER_EVAL, "avg_launch_ms": sweep_avg_ms,
        "note": "frac counts the 7 fp64 operations Eq. 4 asks for per grid point; the kernel executes one "
                "multiply-add and 1.25 other vector instructions per point, see executed_flop_frac and valu_issue_frac",
        # from the instruction counters: fp64 operations executed, as a fraction of the peak
        "executed_flop_frac": (prof["fp64_flops"] / (sweep_avg_ms * 1e-3) / 1e12 / FP64_VECTOR_PEAK_TFLOPS) if prof else None,
        # share of the vector-ALU issue slots of the launch that the scan itself uses: (scan instructions / all vector
        # instructions) x the fraction of cycles the vector ALUs were busy
        "valu_issue_frac": (prof["scan_insts"] / prof["valu_insts"] * prof["valu_busy"]) if prof else None,
    }
    extra["compiler"] = compiler_version()
    extra["kernel_source_sha256"] = kernel_source_digest()
    out = {
        "metric": "(m,s) goodput evals/sec + GA generations/sec; % of FP64 VALU peak",
        "value": evals_per_step * args.steps / elapsed,
        "unit": "evals/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": elapsed * 1e3 / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"{cfg.name}: P={cfg.P} candidates, J={cfg.J} jobs, {cfg.N} nodes x {cfg.cap} GPUs, "
                               f"grid {cfg.Gm}x{cfg.Gs}, p={cfg.p}, fitness + one search step (in place) per step",
                   "evals_per_step": evals_per_step, "generations_per_s": args.steps / elapsed,
                   "generations_per_s_children_only": args.steps / incremental_s,
                   "generations_per_s_changed_rows_only": args.steps / inherited_s},
        "roofline": roofline,
        "extra": extra,
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(wl, cfg)
        import oracle.theta as TH
        tq = time.perf_counter()
        sample = range(0, cfg.J, max(1, cfg.J // 25))
        for j in sample:
            n = records["count"][j]
            TH.fit(*(records[k][j, :n] for k in ("K", "nodes", "m", "s", "T")), n_starts=3)
        out["cpu_baseline"]["theta_fit_seconds_per_job"] = (time.perf_counter() - tq) / len(sample)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
