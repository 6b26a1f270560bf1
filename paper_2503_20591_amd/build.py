"""Compile the HIP library in-tree for gfx950 (cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

PKG = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(PKG, "csrc", "nbos_replay.hip")
LIB = os.path.join(PKG, "libnbos.so")
PROFILE_LIB = os.path.join(PKG, "libnbos_pathprofile.so")      # diagnostic build, see path_profile.py

HIPCC_FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
               "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
               # LDS counters are bumped by one lane on purpose; keep them single ds_add instructions
               "-mllvm", "-amdgpu-atomic-optimizer-strategy=None",
               # a replay is one long dependent chain run by a lone wave: schedule for instruction-level
               # parallelism, not for occupancy (measured: c4 239 -> 230 ms, c3 101 -> 98.8 ms, c2 37.4 -> 36.9 ms)
               "-mllvm", "-amdgpu-sched-strategy=iterative-ilp"]


def _hipcc(out: str, extra: list[str], verbose: bool) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, *extra, "-o", out, SRC]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout + res.stderr)
    if verbose:
        print(" ".join(cmd))
    return out


def build_library(verbose: bool = False) -> str:
    """The product library."""
    return _hipcc(LIB, [], verbose)


def build_profile_library(verbose: bool = False) -> str:
    """The same sources with the path profile compiled in (-DNBOS_PATH_PROFILE): a diagnostic build that
    only `python -m paper_2503_20591_amd.path_profile` loads."""
    return _hipcc(PROFILE_LIB, ["-DNBOS_PATH_PROFILE"], verbose)


if __name__ == "__main__":
    print(build_library(verbose=True))
    print(build_profile_library(verbose=True))
