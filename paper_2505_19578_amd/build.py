"""Compile the HIP library for gfx950 in-tree (hipcc cross-compiles without a GPU)."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "shareprefill.hip")
LIB = os.path.join(HERE, "libshareprefill.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # packed fp32 instructions are kept out of the generated code on purpose
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    # device code never relies on NaN semantics (the score quantiser tests bits); lets fmax chains
    # compile to v_max3 without a canonicalising v_max per operand
    "-Xarch_device", "-fno-honor-nans",
    "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(HERE, "csrc"),
]


def build_library(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc] + HIPCC_FLAGS + [SRC, "-o", LIB]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + res.stdout)
    if verbose:
        print(res.stdout)
    return LIB


def library_path(build_if_missing: bool = True) -> str:
    override = os.environ.get("SHAREPREFILL_LIB")      # an explicitly chosen build of the same library
    if override:
        if not os.path.exists(override):
            raise FileNotFoundError(override)
        return override
    if not os.path.exists(LIB):
        if not build_if_missing:
            raise FileNotFoundError(LIB)
        build_library()
    return LIB


if __name__ == "__main__":
    print(build_library(verbose=True))
