"""Builds ``libmxc.so`` (HIP kernels + C ABI) for gfx950 with hipcc, in-tree."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "csrc", "mxc.hip")
DEPS = [SRC, os.path.join(HERE, "csrc", "mxc_kernels.hpp"), os.path.join(ROOT, "include", "mxc.h")]
LIB = os.path.join(HERE, "libmxc.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # the oracle's arithmetic has no fused multiply-adds; the kernels say so where they want one
    "-ffp-contract=off",
    # never let the compiler form packed-fp32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wextra",
]


def build(force: bool = True) -> str:
    """Compile the library.  With ``force=False`` an up-to-date library is kept."""
    if not force and os.path.exists(LIB) and \
            all(os.path.getmtime(LIB) >= os.path.getmtime(d) for d in DEPS):
        return LIB
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    cmd = [hipcc, *HIPCC_FLAGS, "-I", os.path.join(ROOT, "include"), "-o", LIB + ".tmp", SRC]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout + proc.stderr)
    os.replace(LIB + ".tmp", LIB)
    return LIB


SWEEP_SRC = os.path.join(HERE, "csrc", "sweep.hip")
SWEEP_BIN = os.path.join(HERE, "mxc_sweep")


def build_sweep() -> str:
    """Compile the variant-timing tool ``mxc_sweep`` (optional; the library does not need it)."""
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    flags = [f for f in HIPCC_FLAGS if f not in ("-fPIC", "-shared")]
    cmd = [hipcc, *flags, "-I", os.path.join(ROOT, "include"), "-o", SWEEP_BIN, SWEEP_SRC]
    proc = subprocess.run(cmd, capture_output=True, text=True)
    if proc.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + proc.stdout + proc.stderr)
    return SWEEP_BIN


if __name__ == "__main__":
    import sys
    print(build())
    if "--sweep" in sys.argv:
        print(build_sweep())
