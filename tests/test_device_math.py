"""Error of the fp64 polynomial kernels used on the GPU (exp, log1p, log and the
factored form of Eq. 10), measured on the host against long-double libm.  The
same header is compiled for the device; only the reciprocal seed, ldexp, frexp
and rounding primitives differ."""
import ctypes
import os
import subprocess

import numpy as np
import pytest

HERE = os.path.dirname(os.path.abspath(__file__))


@pytest.fixture(scope="module")
def host_math(tmp_path_factory):
    so = str(tmp_path_factory.mktemp("pxmath") / "libpxmath.so")
    subprocess.run(["g++", "-std=c++17", "-O2", "-ffp-contract=off", "-shared", "-fPIC", "-o", so,
                    os.path.join(HERE, "device_math_host.cpp")], check=True)
    L = ctypes.CDLL(so)
    L.px_host_max_ulp.restype = ctypes.c_double
    L.px_host_max_ulp.argtypes = [ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_long]
    L.px_host_eval.restype = ctypes.c_double
    L.px_host_eval.argtypes = [ctypes.c_int, ctypes.c_double, ctypes.c_double, ctypes.c_double]
    return L


def max_ulp(L, which, x, y=None, g=None):
    x = np.ascontiguousarray(x, np.float64)
    y = np.ascontiguousarray(x if y is None else y, np.float64)
    g = np.ascontiguousarray(np.ones_like(x) if g is None else g, np.float64)
    p = lambda a: a.ctypes.data_as(ctypes.c_void_p)
    return L.px_host_max_ulp(which, p(x), p(y), p(g), x.size)


def test_exp_of_non_positive_arguments(host_math):
    rng = np.random.default_rng(0)
    x = np.concatenate([-rng.uniform(0, 40, 400000), -np.exp(rng.uniform(-30, 6.5, 200000)), rng.uniform(0, 0.7, 100000)])
    assert max_ulp(host_math, 0, x) < 1.0
    assert host_math.px_host_eval(0, 0.0, 0, 1) == 1.0
    assert host_math.px_host_eval(0, -np.inf, 0, 1) == 0.0
    assert host_math.px_host_eval(0, -1000.0, 0, 1) == 0.0


def test_log1p_on_the_unit_interval(host_math):
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.uniform(0, 1, 500000), np.exp(rng.uniform(-40, 0, 200000)), [0.0, 1.0, 0.41421356237309503]])
    assert max_ulp(host_math, 1, x) < 2.5
    assert host_math.px_host_eval(1, 0.0, 0, 1) == 0.0


def test_log_of_positive_numbers(host_math):
    rng = np.random.default_rng(2)
    x = np.concatenate([np.exp(rng.uniform(-20, 20, 500000)), rng.uniform(0.5, 2.0, 300000), [1.0]])
    assert max_ulp(host_math, 2, x) < 2.5
    assert host_math.px_host_eval(2, 1.0, 0, 1) == 0.0


def test_factored_overlap_term_matches_the_direct_power_form(host_math):
    """max(a,b) * exp(log1p(exp(-g|ln a - ln b|))/g) against (a^g + b^g)^(1/g) in long double."""
    rng = np.random.default_rng(3)
    n = 500000
    tg = np.exp(rng.uniform(np.log(1e-3), np.log(10.0), n))
    ts = np.exp(rng.uniform(np.log(1e-3), np.log(10.0), n))
    g = rng.uniform(1.0, 10.0, n)
    assert max_ulp(host_math, 3, tg, ts, g) < 8.0
    # nearly equal terms with the largest exponent are the worst case
    ts2 = tg * (1 + rng.uniform(-1e-3, 1e-3, n))
    assert max_ulp(host_math, 3, tg, ts2, np.full(n, 10.0)) < 8.0
