"""Builds libgact.so (HIP kernels + C ABI) in-tree with hipcc for gfx950."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libgact.so")
SOURCES = [os.path.join(CSRC, "gact_kernels.hip"), os.path.join(CSRC, "gact_reduce.hip"),
           os.path.join(CSRC, "gact_copy.hip"),
           os.path.join(CSRC, "gact_api.cpp"), os.path.join(CSRC, "gact_host.cpp")]

# standalone measurement tool, not part of the library
PROBE = os.path.join(HERE, "traffic_probe.bin")
PROBE_SOURCE = os.path.join(CSRC, "traffic_probe.hip")

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950",
    "-ffp-contract=off",                 # the contract rounds every operation on its own
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-fPIC", "-shared", "-fvisibility=default",
    "-Wall", "-Wno-unused-command-line-argument",
    "-I", os.path.join(ROOT, "include"), "-I", CSRC,
]


def build(verbose: bool = False) -> str:
    """Always compiles; returns the path of the shared library."""
    tmp = LIB + ".tmp%d" % os.getpid()
    cmd = [HIPCC, *FLAGS, "-x", "hip", *SOURCES, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, LIB)
    build_probe(verbose)
    return LIB


def build_probe(verbose: bool = False) -> str:
    """The HBM traffic-ceiling probe bench.py runs beside the workload."""
    tmp = PROBE + ".tmp%d" % os.getpid()
    cmd = [HIPCC, "-O3", "-std=c++17", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang",
           "-packed-fp32-ops", "-Wall", "-Wno-unused-command-line-argument", "-x", "hip", PROBE_SOURCE, "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.check_call(cmd)
    os.replace(tmp, PROBE)
    return PROBE


if __name__ == "__main__":
    print(build(verbose=True))
