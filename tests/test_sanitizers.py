"""The CPU oracle and the library's host code under AddressSanitizer and UndefinedBehaviorSanitizer: one native
program (tests/sanitize/driver.cpp) built from the sources themselves runs round trips, packer-equals-oracle
comparisons, corrupted containers and bad arguments; any report fails the test."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FLAGS = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined", "-fno-sanitize-recover=all"]


def test_oracle_and_host_code_under_asan_and_ubsan(tmp_path):
    csrc = os.path.join(ROOT, "paper_2406_06237_amd", "csrc")
    inc = ["-I", os.path.join(ROOT, "include"), "-I", csrc]
    orc_o, host_o, drv_o, exe = (str(tmp_path / n) for n in ("orc.o", "host.o", "drv.o", "san_driver"))
    try:
        subprocess.check_call(["gcc", "-std=c11", "-ffp-contract=off", *FLAGS, "-c", os.path.join(ROOT, "oracle", "ans_oracle.c"), "-o", orc_o])
        subprocess.check_call(["g++", "-std=c++17", *FLAGS, *inc, "-c", os.path.join(csrc, "anszp_host.cpp"), "-o", host_o])
        subprocess.check_call(["g++", "-std=c++17", *FLAGS, *inc, "-c", os.path.join(ROOT, "tests", "sanitize", "driver.cpp"), "-o", drv_o])
        subprocess.check_call(["g++", *FLAGS, orc_o, host_o, drv_o, "-o", exe, "-lpthread", "-lm"])
    except (subprocess.CalledProcessError, FileNotFoundError) as e:      # no sanitizer runtime in this toolchain
        pytest.skip(f"cannot build with sanitizers: {e}")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    env.pop("LD_PRELOAD", None) if False else None
    r = subprocess.run([exe], capture_output=True, text=True, timeout=600, env=env)
    assert r.returncode == 0 and r.stdout.startswith("ok "), r.stdout + r.stderr[-4000:]
