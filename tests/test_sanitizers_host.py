"""Sanitizer runs of the host-side code (CPU only): the C oracle and the library's planning code are built
with -fsanitize=address,undefined; the oracle's pins then run against that build, and a host driver sweeps
seeded random and extreme shapes through every plan function.  (The kernels and the C ABI's argument path
run under AddressSanitizer in test_emu_kernels.py.)"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    path = subprocess.run(["gcc", "-print-file-name=" + name], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(path) or not os.path.exists(path):
        pytest.skip("no %s next to gcc" % name)
    return path


def test_oracle_pins_under_address_and_ub_sanitizers():
    asan = _runtime("libasan.so")
    env = dict(os.environ, CHEBYKAN_ORACLE_SANITIZE="1", LD_PRELOAD=asan,
               ASAN_OPTIONS="detect_leaks=0:abort_on_error=1", UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1",
               OMP_NUM_THREADS="4")
    pins = ["tests/test_oracle_pins.py", "tests/test_oracle_lut_pins.py", "tests/test_oracle_bases_pins.py"]
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *pins], cwd=ROOT, env=env,
                       capture_output=True, text=True, timeout=1500)
    tail = (r.stdout[-3000:], r.stderr[-3000:])
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, tail


def test_plan_code_under_address_and_ub_sanitizers(tmp_path):
    exe = str(tmp_path / "plans_driver")
    subprocess.run(["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
                    "-fno-omit-frame-pointer", os.path.join(ROOT, "tests", "san", "plans_driver.cpp"), "-o", exe],
                   check=True, cwd=ROOT)
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600)
    assert r.returncode == 0 and "all invariants hold" in r.stdout, (r.stdout[-2000:], r.stderr[-4000:])
    assert "runtime error" not in r.stderr
