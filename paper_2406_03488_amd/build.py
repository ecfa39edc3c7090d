"""Builds libs1f.so (HIP kernels + C ABI) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
INCLUDE = os.path.join(os.path.dirname(HERE), "include")
LIB = os.path.join(HERE, "libs1f.so")
PROBE_LIB = os.path.join(HERE, "libs1f_probe.so")   # measurement aid used by bench.py only

SOURCES = ["s1f_api.hip", "s1f_cache.hip", "s1f_partition.cpp", "s1f_schedule.cpp", "s1f_pipeline.cpp"]
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared", "-Wall",
         # packed fp32 VALU forms are kept out of generated code on this target
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *FLAGS, f"-I{INCLUDE}", f"-I{CSRC}", "-o", LIB, *[os.path.join(CSRC, s) for s in SOURCES]]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout + proc.stderr)
    if verbose:
        print(proc.stderr)
    cmd = [hipcc, *FLAGS, "-o", PROBE_LIB, os.path.join(CSRC, "mfma_peak.hip")]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout + proc.stderr)
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
