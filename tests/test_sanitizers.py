"""CPU sanitizer builds (no GPU): the C oracle and the host-side validation of the C-ABI entry
points, each built with -fsanitize=address,undefined into a small program of its own and run; a
sanitizer report or a wrong answer fails the test."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = os.path.join(ROOT, "tests", "sanitize")


def _run(cmd, exe, tmp_path):
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr[-3000:]
    env = dict(os.environ)
    env.pop("LD_PRELOAD", None)          # the sanitizer runtime must come first in the library list
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "2"
    run = subprocess.run([exe], capture_output=True, text=True, env=env, cwd=str(tmp_path), timeout=300)
    assert run.returncode == 0, (run.stdout + run.stderr)[-3000:]
    assert "runtime error" not in run.stderr and "AddressSanitizer" not in run.stderr, run.stderr[-3000:]
    return run.stdout


def test_oracle_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    cmd = ["gcc", "-O1", "-g", "-std=c99", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
           "-fsanitize=address,undefined", "-fno-omit-frame-pointer", "-static-libasan",
           os.path.join(ROOT, "oracle", "stree_oracle.c"), os.path.join(SAN, "oracle_driver.c"), "-o", exe, "-lm"]
    out = _run(cmd, exe, tmp_path)
    assert out.count("status 0") == 4, out


@pytest.mark.skipif(shutil.which("hipcc") is None and not os.path.exists("/opt/rocm/bin/hipcc"), reason="no hipcc")
def test_host_validation_under_address_and_ub_sanitizers(tmp_path):
    """api.hip (host pass only: validation and dispatch) against stand-in launchers."""
    hipcc = shutil.which("hipcc") or "/opt/rocm/bin/hipcc"
    exe = str(tmp_path / "api_san")
    cmd = [hipcc, "--cuda-host-only", "-O1", "-g", "-std=c++17", "-x", "hip",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined", "-fno-omit-frame-pointer",
           os.path.join(ROOT, "paper_2505_14969_amd", "csrc", "api.hip"), os.path.join(SAN, "api_driver.cpp"),
           "-o", exe]
    out = _run(cmd, exe, tmp_path)
    assert "0 mismatches, 0 launches" in out, out
