"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, no GPU code).

The model compiler (forest_pack.cpp, forest_api_host.cpp) and the C oracle are compiled with the
host compiler and -fsanitize=address,undefined and driven by tests/sanitizer_driver.cpp through
valid models of every shape, every error path, the documented limits and the worked example.  A
sanitizer report or a failed expectation ends the driver with a non-zero status."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2301_13441_amd", "csrc")
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan",
       "-fno-omit-frame-pointer", "-g", "-O1"]


def test_model_compiler_and_oracle_under_asan_ubsan(tmp_path):
    exe = str(tmp_path / "sanitizer_driver")
    oracle_obj = str(tmp_path / "forest_oracle.o")
    subprocess.run(["gcc", "-std=c11", "-c", *[f for f in SAN if not f.startswith("-static")], "-pthread",
                    os.path.join(ROOT, "oracle", "forest_oracle.c"), "-o", oracle_obj], check=True)
    subprocess.run(["g++", "-std=c++17", "-Wall", *SAN, "-pthread",
                    os.path.join(ROOT, "tests", "sanitizer_driver.cpp"),
                    os.path.join(CSRC, "forest_pack.cpp"), os.path.join(CSRC, "forest_api_host.cpp"),
                    oracle_obj, "-lm", "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    run = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=300)
    assert run.returncode == 0, run.stdout + run.stderr
    assert "sanitizer driver: ok" in run.stdout
