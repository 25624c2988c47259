"""Compile the HIP library for gfx950 (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
SOURCE = os.path.join(_HERE, "csrc", "spdy_dp.hip")
INCLUDE = os.path.join(_ROOT, "include")
LIB_PATH = os.path.join(_HERE, "libspdy_dp.so")
PROBE_SOURCE = os.path.join(_HERE, "csrc", "peaks_probe.hip")
PROBE_PATH = os.path.join(_HERE, "peaks_probe")

# packed-fp32 instructions are switched off on purpose (every fp32 op is an ordinary
# v_add_f32 / v_cmp / v_cndmask); subnormals stay on (the default for fp32 on gfx9).
HIPCC_FLAGS = [
    "-O3", "--offload-arch=gfx950", "-std=c++17", "-fPIC",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fno-fast-math", "-ffp-contract=off", "-fno-gpu-flush-denormals-to-zero",
    "-Wall", "-Wextra",
]


def build_library(verbose: bool = False) -> str:
    """Always recompiles; returns the path of the shared library."""
    tmp = LIB_PATH + f".tmp{os.getpid()}"
    cmd = ["hipcc", *HIPCC_FLAGS, "-shared", f"-I{INCLUDE}", SOURCE, "-o", tmp]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout + res.stderr)
    if verbose and res.stderr:
        print(res.stderr)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


def build_probe() -> str:
    """Compile the stand-alone VALU / LDS / bare-sweep rate probe (an executable; bench.py runs
    it as a child process and reports its figures beside the nominal peaks)."""
    tmp = PROBE_PATH + f".tmp{os.getpid()}"
    cmd = ["hipcc", *HIPCC_FLAGS, PROBE_SOURCE, "-o", tmp]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + " ".join(cmd) + "\n" + res.stdout + res.stderr)
    os.replace(tmp, PROBE_PATH)
    return PROBE_PATH


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_probe())
