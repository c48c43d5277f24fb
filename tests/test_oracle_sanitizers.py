"""The CPU checker and the input generator under AddressSanitizer and UndefinedBehaviorSanitizer.

A small C driver (tests/sanitize/driver.c) links oracle/pollux_ref.c and workloads/popgen.c, built with
-fsanitize=address,undefined, and runs fitness calls and search steps on small and ragged shapes with
buffers of exactly the documented sizes.  Any report from either sanitizer fails the test."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_checker_and_generator_are_clean_under_asan_and_ubsan():
    sources = [os.path.join(ROOT, "oracle", "pollux_ref.c"), os.path.join(ROOT, "workloads", "popgen.c"),
               os.path.join(ROOT, "tests", "sanitize", "driver.c")]
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "sanitize_driver")
        # the sanitizer runtimes are linked statically: the process may run with other preloaded libraries
        build = subprocess.run(["gcc", "-std=c11", "-O1", "-g", "-fno-omit-frame-pointer", "-ffp-contract=off", "-fopenmp",
                                "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-static-libasan",
                                "-static-libubsan", "-Wall", "-o", exe] + sources + ["-lm"], capture_output=True, text=True)
        assert build.returncode == 0, build.stderr
        env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0:halt_on_error=1",
                   UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1", OMP_NUM_THREADS="4")
        run = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr and "LeakSanitizer" not in run.stderr, run.stderr
    lines = [ln for ln in run.stdout.splitlines() if ln.startswith("P=")]
    assert len(lines) == 9
    for ln in lines:
        assert float(ln.split("fitness sum")[1].split()[0]) == float(ln.split("fitness sum")[1].split()[0])   # not NaN
