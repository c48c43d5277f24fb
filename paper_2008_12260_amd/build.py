"""Compile the HIP library for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libpollux_hip.so")
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
    subprocess.run(cmd, check=True, cwd=save_temps or HERE)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True, save_temps=sys.argv[1] if len(sys.argv) > 1 else None))
