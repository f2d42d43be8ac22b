"""Builds libqv2.so (HIP kernels + C ABI) in-tree for gfx950 with hipcc."""
from __future__ import annotations

import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
CSRC = os.path.join(HERE, "csrc")
LIB = os.path.join(HERE, "libqv2.so")
SOURCES = [os.path.join(CSRC, "qv2_kernels.hip"), os.path.join(CSRC, "qv2_host.cpp")]

# -ffp-contract=off: each fp32 step of the quantizer rounds once.
# packed-fp32-ops is switched off as a target feature (scalar fp32 code only).
FLAGS = ["--offload-arch=gfx950", "-O3", "-std=c++17", "-fPIC", "-shared",
         "-ffp-contract=off", "-fhip-fp32-correctly-rounded-divide-sqrt",
         "-fno-gpu-flush-denormals-to-zero",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
         "-Wall", "-Wno-unused-command-line-argument"]


def build_lib(verbose: bool = False, defines=(), out: str = LIB) -> str:
    """defines: extra -D options (the tuning knobs of csrc/: QV2_BLOCK_READ, QV2_VEC_READ, QV2_NT_LOADS,
    QV2_XCD_BLOCK_READ, ...)."""
    cmd = ["hipcc", *FLAGS, *[f"-D{d}" for d in defines], "-I", os.path.join(ROOT, "include"),
           "-I", CSRC, "-x", "hip", *SOURCES, "-o", out]
    if verbose:
        print(" ".join(cmd), flush=True)
    subprocess.run(cmd, check=True)
    return out


if __name__ == "__main__":
    import argparse
    ap = argparse.ArgumentParser(description="build libqv2.so, or a variant of it for a measurement")
    ap.add_argument("--define", action="append", default=[], metavar="NAME=VALUE",
                    help="extra -D option, e.g. QV2_NT_LOADS=0 (plain instead of non-temporal loads)")
    ap.add_argument("--out", default=LIB, help="output file (default: the in-tree library)")
    a = ap.parse_args()
    build_lib(verbose=True, defines=a.define, out=a.out)
