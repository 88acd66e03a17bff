"""AddressSanitizer + UndefinedBehaviorSanitizer over the two pieces of plain host code: the CPU
oracle (oracle/q8_oracle.c) and the library's host-only translation unit (codebook and table
builder, csrc/q8opt_host.cpp).  Each is compiled from source together with a driver that calls
every entry point on small, ragged and extreme inputs in exactly-sized buffers; any report from
a sanitizer fails the run."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-g", "-O1"]


def run(exe):
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    return subprocess.run([exe], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env)


@pytest.mark.skipif(shutil.which("gcc") is None, reason="needs gcc")
def test_oracle_under_sanitizers(tmp_path):
    exe = str(tmp_path / "oracle_san")
    subprocess.check_call(["gcc", "-std=c11", "-ffp-contract=off", "-fno-fast-math", *SAN,
                           os.path.join(ROOT, "tests", "sanitize_driver.c"), os.path.join(ROOT, "oracle", "q8_oracle.c"),
                           "-o", exe, "-lm"])
    r = run(exe)
    assert r.returncode == 0 and "cases ok" in r.stdout and "runtime error" not in r.stdout, r.stdout[-3000:]


@pytest.mark.skipif(shutil.which("g++") is None, reason="needs g++")
def test_host_translation_unit_under_sanitizers(tmp_path):
    exe = str(tmp_path / "host_san")
    subprocess.check_call(["g++", "-std=c++17", *SAN, "-I" + os.path.join(ROOT, "include"),
                           "-I" + os.path.join(ROOT, "paper_2412_01195_amd", "csrc"),
                           os.path.join(ROOT, "tests", "sanitize_host_driver.cpp"),
                           os.path.join(ROOT, "paper_2412_01195_amd", "csrc", "q8opt_host.cpp"), "-o", exe])
    r = run(exe)
    assert r.returncode == 0 and "lookups ok" in r.stdout and "runtime error" not in r.stdout, r.stdout[-3000:]
