"""Build the HIP library (gfx950) in-tree with hipcc, and the host-only prefix-cache library with g++."""
from __future__ import annotations

import os
import subprocess

_PKG = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_PKG)
CSRC = os.path.join(_PKG, "csrc")
LIB_PATH = os.path.join(_PKG, "libssm_prefill.so")
SOURCES = ["plan.cpp", "api.hip", "scan_valu.hip", "scan_mfma.hip", "state_advance.hip", "conv1d_prefill.hip"]

# packed-fp32 instructions are switched off for all device code
HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def build_library(verbose: bool = False) -> str:
    srcs = [os.path.join(CSRC, s) for s in SOURCES]
    cmd = ["hipcc", *HIPCC_FLAGS, "-I", os.path.join(_ROOT, "include"), "-I", CSRC,
           "-o", LIB_PATH, *srcs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB_PATH


CACHE_LIB_PATH = os.path.join(_PKG, "libprefix_cache.so")


def build_prefix_cache(verbose: bool = False) -> str:
    """The radix-tree bookkeeping is plain host C++: its own library, no GPU code, no dependency on the HIP one."""
    cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wall", "-Wextra", "-ffp-contract=off",
           "-I", os.path.join(_ROOT, "include"), "-o", CACHE_LIB_PATH, os.path.join(CSRC, "prefix_cache.cpp")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return CACHE_LIB_PATH


PEAK_PROBE_PATH = os.path.join(_PKG, "peak_probe")


def build_peak_probe(verbose: bool = False) -> str:
    """Stand-alone measurement of what the GPU sustains on a streaming copy and on dense MFMA loops."""
    cmd = ["hipcc", "--offload-arch=gfx950", "-O3", "-std=c++17", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-o", PEAK_PROBE_PATH, os.path.join(CSRC, "peak_probe.hip")]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return PEAK_PROBE_PATH


if __name__ == "__main__":
    build_library(verbose=True)
    build_prefix_cache(verbose=True)
    build_peak_probe(verbose=True)
