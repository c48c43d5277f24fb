"""Compile the HIP library for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpollux_hip.so")
BUILD_INFO = LIB + ".buildinfo"     # one line: the compiler that built LIB (written beside it, read by bench.py)
SOURCES = ["pollux_api.hip", "pollux_fitness.hip", "pollux_ga.hip", "pollux_theta.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off",                      # multiply-add is fused only where the code says fma()
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-mllvm", "-disable-machine-licm",        # hoisted constants otherwise spill scalar registers in the sweep
    "-Wall", "-Wno-unused-command-line-argument",
]


def build(verbose: bool = False, save_temps: str | None = None) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + [os.path.join(CSRC, s) for s in SOURCES] + ["-o", LIB]
    if save_temps:
        os.makedirs(save_temps, exist_ok=True)
        cmd += ["-save-temps=cwd"]
    if verbose:
        print(" ".join(cmd), flush=True)
    run = subprocess.run(cmd, cwd=save_temps or HERE, stderr=subprocess.PIPE, text=True)
    # The host pass of every source does not know the device feature named above and says so; that one line is
    # dropped (and counted) so that any other diagnostic stands out.
    known = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"
    lines = run.stderr.splitlines()
    other = [ln for ln in lines if ln.strip() != known]
    if other:
        print("\n".join(other), file=sys.stderr, flush=True)
    if verbose and len(other) != len(lines):
        print(f"({len(lines) - len(other)} host-pass notices about -packed-fp32-ops dropped)", flush=True)
    if run.returncode != 0:
        raise subprocess.CalledProcessError(run.returncode, cmd)
    version = subprocess.run([hipcc, "--version"], capture_output=True, text=True).stdout.splitlines()
    with open(BUILD_INFO, "w") as f:
        f.write("; ".join(v for v in version[:2]) + "\n")
    if verbose:
        print("compiler:", "; ".join(v for v in version[:2]), flush=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, save_temps=sys.argv[1] if len(sys.argv) > 1 else None))
