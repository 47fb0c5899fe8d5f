"""CPU sanitizer job (no GPU): the plain-C oracle and the host-only translation unit of the library
(constants from scales, argument checks, kernel plan) built with AddressSanitizer and
UndefinedBehaviorSanitizer and driven by tests/sanitize/host_sanitize.cpp.  The GPU build is never
compiled with sanitizers."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-fopenmp"]


@pytest.mark.skipif(shutil.which("gcc") is None or shutil.which("g++") is None, reason="needs gcc and g++")
def test_host_logic_and_oracle_under_asan_ubsan(tmp_path):
    obj = str(tmp_path / "qflash_oracle.o")
    exe = str(tmp_path / "host_sanitize")
    subprocess.check_call(["gcc", "-std=c11", "-Wall", "-Wextra"] + SAN +
                          ["-c", os.path.join(ROOT, "oracle", "qflash_oracle.c"), "-o", obj])
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra"] + SAN +
                          ["-I", os.path.join(ROOT, "include"), "-I", os.path.join(ROOT, "paper_2604_25306_amd", "csrc"),
                           os.path.join(ROOT, "tests", "sanitize", "host_sanitize.cpp"),
                           os.path.join(ROOT, "paper_2604_25306_amd", "csrc", "qflash_plan.cpp"), obj, "-o", exe])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert res.returncode == 0, res.stdout[-4000:]
    assert "checks passed" in res.stdout and "ERROR" not in res.stdout and "runtime error" not in res.stdout, res.stdout[-4000:]
