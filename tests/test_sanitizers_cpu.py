"""AddressSanitizer + UndefinedBehaviorSanitizer over the code that runs on the host: the C oracle (every entry
point, small ragged inputs with exact-size buffers) and the library's planning code (interval choice, workspace
layout, argument and flag checks; a host-only translation unit).  GPU code cannot run under the sanitizers on
the test machines, so the kernels' bounds are covered by the layout invariants checked here and by the parity
tests."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
       "-fno-omit-frame-pointer", "-g", "-O1"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")


def run(cmd, **kw):
    res = subprocess.run(cmd, capture_output=True, text=True, timeout=600, **kw)
    assert res.returncode == 0, f"{' '.join(cmd)}\n{res.stdout[-4000:]}\n{res.stderr[-4000:]}"
    return res


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    run(["gcc", "-std=c11", "-fopenmp"] + SAN + ["-o", exe, os.path.join(ROOT, "oracle", "semicrf_oracle.c"),
                                                 os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c"), "-lm"])
    res = run([exe], env=ENV)
    assert "ALL OK" in res.stdout and "BAD" not in res.stdout, res.stdout
    assert "ERROR" not in res.stderr and "runtime error" not in res.stderr, res.stderr


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_planning_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    exe = str(tmp_path / "plan_san")
    csrc = os.path.join(ROOT, "paper_2604_18780_amd", "csrc")
    run(["g++", "-std=c++17"] + SAN + ["-I" + csrc, "-I" + os.path.join(ROOT, "include"), "-o", exe,
                                       os.path.join(csrc, "plan.cpp"),
                                       os.path.join(ROOT, "tests", "sanitize", "plan_driver.cpp")])
    res = run([exe], env=ENV)
    assert "ALL OK" in res.stdout, res.stdout
    assert "ERROR" not in res.stderr and "runtime error" not in res.stderr, res.stderr
