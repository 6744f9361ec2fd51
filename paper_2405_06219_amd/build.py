"""Builds libskvq.so (hipcc, gfx950) in-tree.  `python -m paper_2405_06219_amd.build`."""
from __future__ import annotations

import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

PKG = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(PKG)
CSRC = os.path.join(PKG, "csrc")
LIB = os.path.join(PKG, "libskvq.so")

# -packed-fp32-ops is switched off: the compiler must not form packed fp32 instructions.
COMMON = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-I", os.path.join(ROOT, "include"),
          "-I", CSRC, "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
          "-Wno-unused-command-line-argument"]
# (source, object, extra flags).  The quantizer's fp32 operations must each round once.  The
# matrix-core decode kernels are compiled once per (key levels, value levels) pair.
DECODE_FORMATS = [(4, 3), (4, 4), (4, 16), (8, 8), (16, 3), (16, 4), (16, 16)]
UNITS = [
    ("skvq_api.hip", "skvq_api.o", []),
    ("skvq_quantize.hip", "skvq_quantize.o", ["-ffp-contract=off"]),
    ("skvq_decode.hip", "skvq_decode.o", []),
    ("skvq_prefill_attn.hip", "skvq_prefill_attn.o", []),
    ("skvq_calibrate.hip", "skvq_calibrate.o", ["-ffp-contract=off"]),
    ("skvq_reorder.hip", "skvq_reorder.o", ["-ffp-contract=off"]),
    ("skvq_yardstick.hip", "skvq_yardstick.o", []),
    ("skvq_decode_mfma.hip", "skvq_decode_mfma.o", []),
] + [("skvq_decode_mfma_inst.hip", f"skvq_decode_mfma_k{kl}_v{vl}.o", [f"-DSKVQ_KL={kl}", f"-DSKVQ_VL={vl}"])
     for kl, vl in DECODE_FORMATS]
# SKVQ_RESOURCE_USAGE=1 prints each kernel's registers, scratch and LDS
if os.environ.get("SKVQ_RESOURCE_USAGE"):
    COMMON.append("-Rpass-analysis=kernel-resource-usage")


def build(verbose: bool = False) -> str:
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")

    def compile_unit(unit):
        src, obj, extra = unit
        obj = os.path.join(CSRC, obj)
        cmd = [hipcc, *COMMON, *extra, "-c", os.path.join(CSRC, src), "-o", obj]
        if verbose:
            print(" ".join(cmd), flush=True)
        subprocess.run(cmd, check=True)
        return obj

    jobs = max(1, min(len(UNITS), int(os.environ.get("MAX_JOBS", "0")) or (os.cpu_count() or 1), 16))
    with ThreadPoolExecutor(max_workers=jobs) as pool:
        objs = list(pool.map(compile_unit, UNITS))
    cmd = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", LIB, *objs]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return LIB


if __name__ == "__main__":
    print(build(verbose="-q" not in sys.argv))
