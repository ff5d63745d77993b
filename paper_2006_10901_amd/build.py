"""Builds libspdl.so (HIP, gfx950 only) next to this file with hipcc."""
from __future__ import annotations

import glob
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libspdl.so")
CSRC = os.path.join(_HERE, "csrc")
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

# Packed fp32 VALU instructions are switched off for every translation unit.
HIP_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


MICROBENCH_SRC = os.path.join(_HERE, "microbench", "inner_loop_rates.hip")
MICROBENCH_BIN = os.path.join(_HERE, "microbench", "inner_loop_rates")


def build_microbench(verbose: bool = False) -> str:
    """The stand-alone program that measures the issue rates bounding the kernels' inner loops
    (run it on the GPU machine: paper_2006_10901_amd/microbench/inner_loop_rates)."""
    flags = [f for f in HIP_FLAGS if f not in ("-fPIC", "-shared")]
    cmd = [HIPCC, *flags, "-o", MICROBENCH_BIN, MICROBENCH_SRC]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    return MICROBENCH_BIN


CLOCKS_LIB_PATH = os.path.join(_HERE, "microbench", "libspdl_phase_clocks.so")


def build_phase_clocks(verbose: bool = False) -> str:
    """A second copy of the library with clocks compiled into the slab kernels
    (-DSPDL_PHASE_CLOCKS), for microbench/phase_clocks.py only; the product library has none."""
    cmd = [HIPCC, *HIP_FLAGS, "-DSPDL_PHASE_CLOCKS", "-o", CLOCKS_LIB_PATH, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    return CLOCKS_LIB_PATH


def sources():
    return sorted(glob.glob(os.path.join(CSRC, "*.hip")))


def build(verbose: bool = False) -> str:
    cmd = [HIPCC, *HIP_FLAGS, "-o", LIB_PATH, *sources()]
    if verbose:
        print(" ".join(cmd), flush=True)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    return LIB_PATH


if __name__ == "__main__":
    print(build(verbose=True))
    print(build_microbench(verbose=True))
    print(build_phase_clocks(verbose=True))
