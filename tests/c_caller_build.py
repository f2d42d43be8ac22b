"""Compiles tests/abi_c_caller.c (the plain-C caller of the C ABI) with gcc as strict C99."""
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
SRC = os.path.join(HERE, "abi_c_caller.c")
LIBDIR = os.path.join(ROOT, "paper_2501_07161_amd")
ROCM = os.environ.get("ROCM_PATH", "/opt/rocm")
EXE = os.path.join(HERE, "abi_c_caller")          # where __graft_entry__.build() puts it


def build(out: str = EXE) -> str:
    # HIP's headers are taken as system headers: -pedantic then judges qv2.h and the caller only
    cmd = ["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-O1", "-D__HIP_PLATFORM_AMD__",
           "-isystem", os.path.join(ROCM, "include"), "-I", os.path.join(ROOT, "include"), SRC,
           "-L", LIBDIR, "-lqv2", "-L", os.path.join(ROCM, "lib"), "-lamdhip64", "-o", out]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        raise RuntimeError("gcc failed on abi_c_caller.c:\n" + r.stderr[-4000:])
    return out
