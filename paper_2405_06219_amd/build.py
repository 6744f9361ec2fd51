"""Builds libskvq.so (hipcc, gfx950) in-tree.  `python -m paper_2405_06219_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libskvq.so")

# -packed-fp32-ops is switched off: the compiler must not form packed fp32 instructions.
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"),
          "-I", CSRC, "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-command-line-argument"]
# per-file extras: the quantizer's fp32 operations must each round once
SOURCES = {
    "skvq_api.hip": [],
    "skvq_quantize.hip": ["-ffp-contract=off"],
    "skvq_decode.hip": [],
    "skvq_decode_mfma.hip": [],
}
# SKVQ_RESOURCE_USAGE=1 prints each kernel's registers, scratch and LDS
if os.environ.get("SKVQ_RESOURCE_USAGE"):
    COMMON.append("-Rpass-analysis=kernel-resource-usage")


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objs = []
    for src, extra in SOURCES.items():
        obj = os.path.join(CSRC, src.replace(".hip", ".o"))
        cmd = [hipcc, *COMMON, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        objs.append(obj)
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-q" not in sys.argv))
