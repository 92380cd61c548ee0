"""Build the C-ABI library (libtli.so) from csrc/ with hipcc for gfx950, in-tree."""
from __future__ import annotations

import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(_HERE)
SOURCES = [os.path.join(_HERE, "csrc", "tli_kernels.hip"), os.path.join(_HERE, "csrc", "tli_host_map.cpp")]
LIB = os.path.join(_HERE, "libtli.so")

HIPCC_FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    # no implicit a*b+c fusion: the kernels rely on products being rounded exactly where they say so (a chunk's
    # reference must be THE fp32 number the exponents were formed against); wanted FMAs are written as fmaf
    "-ffp-contract=off",
    # packed fp32 instructions are disabled for the device pass (the host pass does not know the feature)
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-I", os.path.join(ROOT, "include"),
]


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    extra = os.environ.get("TLI_HIPCC_EXTRA", "").split()  # e.g. -D switches for kernel experiments
    cmd = [hipcc, *HIPCC_FLAGS, *extra, "-o", LIB, *SOURCES]
    if verbose:
        print(" ".join(cmd))
    res = subprocess.run(cmd, capture_output=True, text=True)
    noise = "is not a recognized feature for this target"
    err = "\n".join(l for l in res.stderr.splitlines() if noise not in l)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed:\n" + err)
    if verbose and err.strip():
        print(err)
    return LIB


if __name__ == "__main__":
    print(build(verbose=True))
