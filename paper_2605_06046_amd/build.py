"""Compiles libfea.so (host bookkeeping + HIP kernels for gfx950) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libfea.so")
SOURCES = ["fea_host.cpp", "fea_cht.cpp", "fea_policy.cpp", "fea_planner.hip", "fea_sweep_generic.hip", "fea_sweep_mfma.hip", "fea_append.hip", "fea_hash.hip", "fea_decode.hip", "fea_decode_static.hip", "fea_calibrate.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops"]


def build(verbose: bool = False) -> str:
    """Always recompiles; returns the path of the shared library."""
    cmd = [HIPCC, *FLAGS, "-o", LIB, *[os.path.join(CSRC, s) for s in SOURCES]]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
