"""Builds librsr.so (HIP, gfx950 only) in-tree with hipcc."""
from __future__ import annotations

import os
import subprocess
import sys

PKG_DIR = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(PKG_DIR, "csrc")
INCLUDE = os.path.join(os.path.dirname(PKG_DIR), "include")
LIB_PATH = os.path.join(PKG_DIR, "librsr.so")
SOURCES = ["rsr_api.hip", "rsr_preprocess.hip", "rsr_matvec.hip", "rsr_dense.hip", "rsr_probe.hip", "rsr_narrow.hip"]

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # the first kernel arguments (stream and vector pointers, geometry) arrive in registers
    # instead of through a scalar load at the start of every wave
    "-mllvm", "-amdgpu-kernarg-preload-count=14",
    "-Wall", "-Wno-unused-command-line-argument",
]


def build_library(verbose: bool = False) -> str:
    """Compile every HIP source into paper_2603_27462_amd/librsr.so."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB_PATH + ".tmp%d" % os.getpid()
    cmd = [hipcc] + HIPCC_FLAGS + ["-I", INCLUDE, "-I", CSRC]
    cmd += [os.path.join(CSRC, s) for s in SOURCES] + ["-o", tmp]
    if verbose:
        print(" ".join(cmd), file=sys.stderr)
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout)
    if verbose and proc.stdout.strip():
        print(proc.stdout, file=sys.stderr)
    os.replace(tmp, LIB_PATH)
    return LIB_PATH


def sources_newer_than_library() -> list:
    """Source files modified after the built library (empty when it is up to date or absent)."""
    if not os.path.exists(LIB_PATH):
        return []
    built = os.path.getmtime(LIB_PATH)
    files = [os.path.join(CSRC, f) for f in sorted(os.listdir(CSRC))]
    files.append(os.path.join(INCLUDE, "rsr.h"))
    return [os.path.relpath(f, os.path.dirname(PKG_DIR)) for f in files
            if f.endswith((".hip", ".h")) and os.path.getmtime(f) > built + 1.0]


if __name__ == "__main__":
    print(build_library(verbose=True))
