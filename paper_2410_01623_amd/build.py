"""Builds the HIP library (libfira.so) for gfx950 in-tree with hipcc.  No GPU needed to build."""
from __future__ import annotations

import os
import shutil
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
LIB_PATH = os.path.join(PKG_DIR, "libfira.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC", "-fvisibility=hidden",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",   # no packed-fp32 code generation
    "-Wno-unused-command-line-argument",
]


def build_library(verbose: bool = True, extra_flags=()) -> str:
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    src = os.path.join(CSRC, "fira.hip")
    cmd = [hipcc, *HIPCC_FLAGS, *extra_flags, src, "-o", LIB_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    # the host pass warns that it does not know the packed-fp32 feature: harmless, filtered out
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err, file=sys.stderr)
    return LIB_PATH


MICROBENCH_PATH = os.path.join(PKG_DIR, "fira_microbench")


def build_microbench(verbose: bool = True) -> str:
    """The machine-calibration program (HBM streams, MFMA rate, LDS read rate); not part of the library."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    flags = [f for f in HIPCC_FLAGS if f not in ("-shared", "-fPIC", "-fvisibility=hidden")]
    cmd = [hipcc, *flags, os.path.join(CSRC, "fira_microbench.hip"), "-o", MICROBENCH_PATH]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if "packed-fp32-ops" not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    return MICROBENCH_PATH


if __name__ == "__main__":
    print(build_library())
    print(build_microbench())
