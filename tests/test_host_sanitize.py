"""Builds csrc/qv2_host.cpp (plan builder, finalize, rank, BOPs, KL, regrouping: everything of
the library that needs no GPU) together with tests/host_checks.cpp under AddressSanitizer and
UndefinedBehaviorSanitizer with g++, and runs it on the CPU.  The program checks the invariants
of the tile tables the kernels rely on over many layer tables (every element covered exactly once
by every pass, partial slots unique and inside the workspace, fold lists complete) and drives the
host functions over random and hostile inputs."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2501_07161_amd", "csrc")


def _build(out, sanitize):
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-Wall", "-Wextra",
           "-I", os.path.join(ROOT, "include"), "-I", CSRC,
           os.path.join(ROOT, "tests", "host_checks.cpp"), os.path.join(CSRC, "qv2_host.cpp"), "-o", out]
    if sanitize:
        cmd[1:1] = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"]
    return subprocess.run(cmd, capture_output=True, text=True)


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_code_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_checks")
    r = _build(exe, True)
    sanitized = r.returncode == 0
    if not sanitized:                       # no sanitizer runtime installed: the checks still run
        r = _build(exe, False)
    assert r.returncode == 0, r.stderr[-3000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe, str(tmp_path)], capture_output=True, text=True, env=env, timeout=600)
    assert run.returncode == 0, (run.stdout + run.stderr)[-3000:]
    assert "host checks ok" in run.stdout
    print("sanitizers:", "address+undefined" if sanitized else "not available, plain build")
