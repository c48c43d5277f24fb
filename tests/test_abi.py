"""The C-ABI library loads, exports every symbol declared in include/pollux.h, and
rejects bad arguments on the host before touching a device (no GPU needed)."""
import ctypes
import os
import re

import pytest

import paper_2008_12260_amd as px

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "pollux.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pollux_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(px.EXPORTS)
    L = px.lib()
    for n in names:
        assert getattr(L, n) is not None
    assert px.version() == 105
    assert px.strerror(0) == "success" and "workspace" in px.strerror(px.PX_E_WORKSPACE)
    assert px.strerror(-99) == "unknown error code"


def test_workspace_size_grows_with_the_problem_and_rejects_bad_dims():
    small = px.workspace_size(px.Dims(16, 8, 4, 32, 8, 0, 0))
    big = px.workspace_size(px.Dims(4096, 1000, 256, 128, 32, 0, 0))
    assert 0 < small < big and small % 256 == 0
    assert big >= 4096 * 1000 * 12
    for bad in (px.Dims(0, 8, 4, 32, 8, 0, 0), px.Dims(16, -1, 4, 32, 8, 0, 0), px.Dims(16, 8, 0, 32, 8, 0, 0),
                px.Dims(16, 8, 4, 32, 8, 7, 0), px.Dims(70000, 70000, 4, 1, 1, 0, 0)):
        with pytest.raises(px.PolluxError) as e:
            px.workspace_size(bad)
        assert e.value.code == px.PX_E_INVALID_ARG


def test_entry_points_reject_bad_arguments_without_a_device():
    L = px.lib()
    d = px.Dims(16, 8, 4, 32, 8, 0, 0)
    fake = ctypes.c_void_p(0x1000)          # never dereferenced: validation fails first
    null = ctypes.c_void_p(0)
    args = [fake] * 6 + [-1.0, 30.0, fake, 1 << 30] + [fake] * 6 + [null]
    assert L.pollux_fitness(None, *args) == px.PX_E_INVALID_ARG
    bad = list(args); bad[0] = null
    assert L.pollux_fitness(ctypes.byref(d), *bad) == px.PX_E_INVALID_ARG
    bad = list(args); bad[6] = float("nan")
    assert L.pollux_fitness(ctypes.byref(d), *bad) == px.PX_E_INVALID_ARG
    bad = list(args); bad[7] = -1.0
    assert L.pollux_fitness(ctypes.byref(d), *bad) == px.PX_E_INVALID_ARG
    bad = list(args); bad[8] = null
    assert L.pollux_fitness(ctypes.byref(d), *bad) == px.PX_E_WORKSPACE
    bad = list(args); bad[8] = ctypes.c_void_p(0x1001)
    assert L.pollux_fitness(ctypes.byref(d), *bad) == px.PX_E_WORKSPACE
    bad = list(args); bad[9] = 16
    assert L.pollux_fitness(ctypes.byref(d), *bad) == px.PX_E_WORKSPACE
    bad = list(args); bad[11] = null                       # best_m without best_s (args[10] is fitness)
    assert L.pollux_fitness(ctypes.byref(d), *bad) == px.PX_E_INVALID_ARG
    bad = list(args); bad[12] = null
    assert L.pollux_fitness(ctypes.byref(d), *bad) == px.PX_E_INVALID_ARG
    d0 = px.Dims(16, 8, 4, 0, 8, 0, 0)
    assert L.pollux_fitness(ctypes.byref(d0), *args) == px.PX_E_INVALID_ARG
    d_big = px.Dims(16, 8, 4, 1 << 20, 1 << 13, 0, 0)       # a job's lane-mask table would pass 2^31 bytes
    assert L.pollux_fitness(ctypes.byref(d_big), *args) == px.PX_E_INVALID_ARG

    ga = px.GaParams(1, 0, 8, 0, 0)
    gargs = [fake, fake, fake, ctypes.byref(ga), fake, 1 << 30, ctypes.c_void_p(0x100000), null]
    bad = list(gargs); bad[6] = fake                       # children alias parents
    assert L.pollux_ga_step(ctypes.byref(d), *bad) == px.PX_E_INVALID_ARG
    ga0 = px.GaParams(1, 0, 0, 0, 0)
    bad = list(gargs); bad[3] = ctypes.byref(ga0)
    assert L.pollux_ga_step(ctypes.byref(d), *bad) == px.PX_E_INVALID_ARG
    ga17 = px.GaParams(1, 0, 17, 0, 0)
    bad = list(gargs); bad[3] = ctypes.byref(ga17)
    assert L.pollux_ga_step(ctypes.byref(d), *bad) == px.PX_E_INVALID_ARG
    bad = list(gargs); bad[4] = null
    assert L.pollux_ga_step(ctypes.byref(d), *bad) == px.PX_E_WORKSPACE
    assert L.pollux_last_status(null, null, None) == px.PX_E_INVALID_ARG


def test_the_entry_point_with_library_owned_scratch_checks_its_limit_on_the_host():
    """pollux_fitness_static: same argument checks as pollux_fitness, and a problem whose scratch need exceeds the
    library's array is refused before any device is touched."""
    L = px.lib()
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    ok = [fake] * 6 + [-1.0, 30.0] + [fake] * 7 + [null]
    big = px.Dims(4096, 1000, 256, 128, 32, 0, 0)
    assert px.workspace_size(big) > px.STATIC_SCRATCH_BYTES
    assert L.pollux_fitness_static(ctypes.byref(big), *ok) == px.PX_E_WORKSPACE
    fits = px.Dims(1000, 200, 64, 64, 16, 0, 0)
    assert px.workspace_size(fits) <= px.STATIC_SCRATCH_BYTES
    bad = list(ok); bad[0] = null
    assert L.pollux_fitness_static(ctypes.byref(fits), *bad) == px.PX_E_INVALID_ARG
    bad = list(ok); bad[6] = float("inf")
    assert L.pollux_fitness_static(ctypes.byref(fits), *bad) == px.PX_E_INVALID_ARG
    bad = list(ok); bad[7] = -1.0
    assert L.pollux_fitness_static(ctypes.byref(fits), *bad) == px.PX_E_INVALID_ARG
    assert L.pollux_fitness_static(None, *ok) == px.PX_E_INVALID_ARG
    text = open(os.path.join(ROOT, "include", "pollux.h")).read()
    assert f"#define POLLUX_STATIC_SCRATCH_BYTES ({px.STATIC_SCRATCH_BYTES >> 20}u << 20)" in text


def test_the_newer_entry_points_reject_bad_arguments_without_a_device():
    L = px.lib()
    fake, null = ctypes.c_void_p(0x1000), ctypes.c_void_p(0)
    ok_fit = [4, 8] + [fake] * 6 + [null, 100, 3, fake, fake, null, null]
    for pos, value in ((0, 0), (1, 0), (9, -1), (10, 0), (10, 6), (2, null), (7, null), (11, null), (12, null)):
        bad = list(ok_fit)
        bad[pos] = value
        assert L.pollux_fit_theta(*bad) == px.PX_E_INVALID_ARG, pos
    d = px.Dims(1, 8, 1, 32, 8, 0, 0)
    ws = px.workspace_size(d)
    assert L.pollux_goodput_per_gpu(ctypes.byref(d), fake, fake, 0, 4, fake, ws, fake, null) == px.PX_E_INVALID_ARG
    assert L.pollux_goodput_per_gpu(ctypes.byref(d), fake, fake, 4, 0, fake, ws, fake, null) == px.PX_E_INVALID_ARG
    assert L.pollux_goodput_per_gpu(ctypes.byref(d), fake, fake, 4, 4, fake, ws, null, null) == px.PX_E_INVALID_ARG
    assert L.pollux_goodput_per_gpu(ctypes.byref(d), fake, fake, 4, 4, fake, ws - 1, fake, null) == px.PX_E_WORKSPACE
    flagged = px.Dims(1, 8, 1, 32, 8, 0, px.PX_FLAG_MEMOISE)
    assert L.pollux_goodput_per_gpu(ctypes.byref(flagged), fake, fake, 4, 4, fake, ws, fake, null) == px.PX_E_INVALID_ARG
    assert L.pollux_autoscale(0, 4, fake, fake, 0.6, 0.5, fake, null) == px.PX_E_INVALID_ARG
    assert L.pollux_autoscale(8, 4, fake, fake, float("inf"), 0.5, fake, null) == px.PX_E_INVALID_ARG
    assert L.pollux_autoscale(8, 4, null, fake, 0.6, 0.5, fake, null) == px.PX_E_INVALID_ARG
    tick = [ctypes.byref(d)] + [fake] * 6 + [60.0, 30.0, fake, ws, fake, fake, fake, null]
    for pos, value in ((7, -1.0), (8, float("nan")), (3, null), (11, null), (13, null)):
        bad = list(tick)
        bad[pos] = value
        assert L.pollux_sim_tick(*bad) == px.PX_E_INVALID_ARG, pos
    sampled = px.Dims(16, 8, 4, 32, 8, 1, px.PX_FLAG_SAMPLE_M)        # the sampling argmax exists in fp64 only
    with pytest.raises(px.PolluxError):
        px.workspace_size(sampled)
    ga = px.GaParams(1, 0, 8, 0, 2)                                    # unknown search flag
    dd = px.Dims(16, 8, 4, 32, 8, 0, 0)
    assert L.pollux_ga_step(ctypes.byref(dd), fake, fake, fake, ctypes.byref(ga), fake, 1 << 30, ctypes.c_void_p(0x90000000), null) == px.PX_E_INVALID_ARG
    # pollux_generation: in place always; rows are inherited only in place, and of a memoised call only when it was
    # asked to leave its per-pair results in the workspace
    def generation(dims, flags):
        g = px.GaParams(1, 0, 8, 0, flags, None)
        return L.pollux_generation(ctypes.byref(dims), *([fake] * 6), -1.0, 30.0, ctypes.byref(g), null, 0, *([fake] * 6), null)
    assert generation(dd, 0) == px.PX_E_INVALID_ARG
    assert generation(dd, px.PX_GA_INHERIT_ROWS) == px.PX_E_INVALID_ARG
    assert generation(dd, px.PX_GA_IN_PLACE | 4) == px.PX_E_INVALID_ARG
    memo = px.Dims(16, 8, 4, 32, 8, 0, px.PX_FLAG_MEMOISE)
    assert generation(memo, px.PX_GA_IN_PLACE | px.PX_GA_INHERIT_ROWS) == px.PX_E_INVALID_ARG
    # (valid flags get as far as the workspace check)
    assert generation(dd, px.PX_GA_IN_PLACE) == px.PX_E_WORKSPACE
    assert generation(dd, px.PX_GA_IN_PLACE | px.PX_GA_INHERIT_ROWS) == px.PX_E_WORKSPACE
    memo_pairs = px.Dims(16, 8, 4, 32, 8, 0, px.PX_FLAG_MEMOISE | px.PX_FLAG_PAIR_RESULTS)
    assert generation(memo_pairs, px.PX_GA_IN_PLACE | px.PX_GA_INHERIT_ROWS) == px.PX_E_WORKSPACE


def test_shapes_whose_bookkeeping_does_not_fit_on_chip_are_rejected():
    fake, null = ctypes.c_void_p(0x100000), ctypes.c_void_p(0)
    ga = px.GaParams(1, 0, 1, 0, 0, None)
    for J, N, ok in ((1000, 5000, True), (1000, 5400, False), (8, 6000, True), (8, 6600, False), (7000, 256, True), (8000, 256, False)):
        d = px.Dims(2, J, N, 1, 1, 0, 0)
        rc = px.lib().pollux_ga_step(ctypes.byref(d), fake, fake, fake, ctypes.byref(ga), null, 0, ctypes.c_void_p(0x7f0000000000), null)
        # a shape that fits gets as far as the workspace check; one that does not is refused before it
        assert rc == (px.PX_E_WORKSPACE if ok else px.PX_E_INVALID_ARG), (J, N, rc)
