"""The C oracle and the host-side slot bookkeeping once under AddressSanitizer and
UndefinedBehaviorSanitizer (CPU builds of small drivers in tests/sanitize/)."""
import os
import shutil
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(HERE)
# the sanitizer runtimes are linked statically, so their place in the process's library list does
# not depend on what else the environment loads
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1", "-static-libasan",
       "-static-libubsan"]


def build_and_run(tmp_path, compiler, sources, extra):
    if shutil.which(compiler) is None:
        pytest.skip(f"{compiler} not installed")
    exe = str(tmp_path / "driver")
    res = subprocess.run([compiler, *SAN, *extra, "-o", exe, *sources], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1", OMP_NUM_THREADS="4")
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=120)
    assert res.returncode == 0 and res.stdout.strip() == "ok", res.stdout + res.stderr


def test_oracle_under_asan_ubsan(tmp_path):
    build_and_run(tmp_path, "gcc", [os.path.join(HERE, "sanitize", "oracle_san.c"), os.path.join(ROOT, "oracle", "ifx_oracle.c")],
                  ["-fopenmp", "-lm"])


def test_ring_under_asan_ubsan(tmp_path):
    build_and_run(tmp_path, "g++", [os.path.join(HERE, "sanitize", "ring_san.cpp")], ["-std=c++17"])
