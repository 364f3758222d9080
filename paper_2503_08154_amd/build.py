"""Compile the HIP library (libs2a.so) in-tree for gfx950.

    python -m paper_2503_08154_amd.build

The shared object lands next to the sources' package so that it travels with
the tree; nothing is installed into site-packages.
"""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libs2a.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950",
    "-O3",
    "-std=c++17",
    "-fPIC",
    "-shared",
    "-fno-gpu-flush-denormals-to-zero",   # y below 2^-126 must come out as denormals
    "-ffp-contract=off",                  # FMAs only where the source writes them
    # no packed-fp32 VALU forms (v_pk_add/mul/fma_f32) in the device code.  The device pass honours
    # the feature switch; the host pass of the same command does not know it and prints one
    # warning per pass, which is dropped below by exact match.  tests/test_build.py compiles the
    # device code to assembly and checks that none of these instructions is in it.
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wno-unused-command-line-argument",
]


HOST_PASS_WARNING = "'-packed-fp32-ops' is not a recognized feature for this target (ignoring feature)"


def device_assembly(out_path: str) -> str:
    """Compile only the device code of the library to gfx950 assembly text (for checks on the
    generated instructions); returns out_path."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    cmd = [hipcc, *flags, "--cuda-device-only", "-S", "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(CSRC, "s2a_api.hip"), "-o", out_path]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        sys.stderr.write(res.stderr + "\n")
        raise RuntimeError("hipcc failed")
    return out_path


def build_library(verbose: bool = True) -> str:
    """Always recompiles; returns the path of the shared library."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    tmp = LIB + f".{os.getpid()}.tmp"
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(CSRC, "s2a_api.hip"), "-o", tmp]
    if verbose:
        print(" ".join(cmd), flush=True)
    res = subprocess.run(cmd, capture_output=True, text=True)
    err = "\n".join(l for l in res.stderr.splitlines() if l.strip() != HOST_PASS_WARNING)
    if res.returncode != 0:
        sys.stderr.write(err + "\n")
        raise RuntimeError("hipcc failed")
    if verbose and err.strip():
        sys.stderr.write(err + "\n")
    os.replace(tmp, LIB)
    return LIB


if __name__ == "__main__":
    print(build_library())
