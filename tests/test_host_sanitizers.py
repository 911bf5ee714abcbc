"""Host-side code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only): the C oracle
(oracle/tva_oracle.c) and the host part of the library (csrc/cast.cpp: tree-size selection with its
caller-owned state block, the host mask builder) are compiled with -fsanitize=address,undefined into one
small program (tests/sanitize/host_driver.cpp) whose buffers have exactly the documented sizes, and run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_and_host_code_are_clean_under_asan_and_ubsan(tmp_path):
    gxx, gcc = shutil.which("g++"), shutil.which("gcc")
    if not gxx or not gcc:
        pytest.skip("no host compiler")
    san = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan", "-g", "-O1", "-fopenmp"]
    inc = ["-I", os.path.join(ROOT, "include")]
    obj = str(tmp_path / "oracle.o")
    exe = str(tmp_path / "host_driver")
    subprocess.run([gcc, *san, "-c", os.path.join(ROOT, "oracle", "tva_oracle.c"), "-o", obj], check=True)
    subprocess.run([gxx, *san, "-std=c++17", *inc, os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp"),
                    os.path.join(ROOT, "paper_2510_26577_amd", "csrc", "cast.cpp"), obj, "-lm", "-o", exe], check=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
               OMP_NUM_THREADS="2")
    env.pop("LD_PRELOAD", None)     # the sanitizer runtime has to come first in the process
    res = subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.PIPE, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "AddressSanitizer" not in res.stderr and "runtime error" not in res.stderr, res.stderr
    assert "0 failure(s)" in res.stdout
