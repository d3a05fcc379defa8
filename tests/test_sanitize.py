"""Host-only sanitizer builds (address + undefined behaviour) of the oracle's C code and of the
planner behind the C ABI, each driven by a shape fuzz (tests/sanitize/).  No GPU, no HIP: the
planner's sources (plan.cpp, setup.cpp) are plain C++ and the kernel launchers are stubbed."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1",
       "-static-libasan"]
# the test harness may preload a library of its own before the sanitizer's runtime
ENV = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1:abort_on_error=0",
           UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")


def _build_and_run(tmp_path, compiler, sources, extra, args):
    exe = str(tmp_path / "fuzz")
    cmd = [compiler] + SAN + extra + sources + ["-o", exe, "-lm"]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-4000:]
    run = subprocess.run([exe] + args, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=ENV,
                         timeout=600)
    assert run.returncode == 0, run.stdout[-4000:]
    assert "ERROR" not in run.stdout and "runtime error" not in run.stdout, run.stdout[-4000:]
    return run.stdout


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_planner_under_sanitizers(tmp_path):
    csrc = os.path.join(ROOT, "paper_2002_00552_amd", "csrc")
    out = _build_and_run(tmp_path, "g++",
                         [os.path.join(ROOT, "tests", "sanitize", "planner_fuzz.cpp"),
                          os.path.join(csrc, "plan.cpp"), os.path.join(csrc, "setup.cpp")],
                         ["-std=c++17", "-Wall"], ["1500"])
    assert "planner fuzz:" in out


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_sanitizers(tmp_path):
    out = _build_and_run(tmp_path, "gcc", [os.path.join(ROOT, "tests", "sanitize", "oracle_fuzz.c")],
                         ["-std=c99", "-Wall", "-fopenmp"], ["150"])
    assert "oracle fuzz:" in out
