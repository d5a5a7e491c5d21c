"""Builds libarcq.so (hand-written HIP for gfx950) in-tree with hipcc.

    python -m paper_2601_07475_amd.build

Flags: -ffp-contract=off and correctly rounded fp32 division keep the quantizer's
arithmetic one-rounding-per-step; packed fp32 VALU ops are disabled.
"""
import os
import shutil
import subprocess
import sys

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libarcq.so")
SOURCES = ["api.hip", "quantize.hip", "gemm.hip", "gemm_ksplit.hip", "check_perm.hip", "calibrate.hip", "mx_quantize.hip", "mx_gemm.hip", "probe.hip"]

FLAGS = [
    "--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
    "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
    "-Wall", "-Wno-unused-function",
]


def hipcc():
    exe = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    if not os.path.exists(exe):
        raise RuntimeError("hipcc not found")
    return exe


def build(verbose=True, extra=()):
    cmd = [hipcc(), *FLAGS, *extra, *[os.path.join(CSRC, s) for s in SOURCES], "-o", LIB]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True, cwd=HERE)
    return LIB


if __name__ == "__main__":
    build(extra=sys.argv[1:])
