"""Builds the HIP library in-tree: paper_2601_20499_amd/libdf_hip.so (gfx950 only)."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libdf_hip.so")
SOURCES = ["df_host.cpp", "df_cache.hip", "df_attn.hip"]


def hipcc_command(out: str = LIB, extra=()):
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, "--offload-arch=gfx950", "-O3", "-std=c++17", "-shared", "-fPIC",
           # packed fp32 VALU forms are kept out of the generated code on purpose
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Wno-unused-command-line-argument", "-Wno-unknown-warning-option",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC]
    cmd += list(extra)
    for s in SOURCES:
        path = os.path.join(CSRC, s)
        cmd += (["-x", "hip", path] if s.endswith(".hip") else ["-x", "c++", path])
    cmd += ["-o", out]
    return cmd


def build_library(verbose: bool = True, extra=()) -> str:
    cmd = hipcc_command(extra=extra)
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, cwd=CSRC)
    return LIB


if __name__ == "__main__":
    build_library(extra=sys.argv[1:])
