"""The CPU oracle and the host side of libzipccl.so under AddressSanitizer + UndefinedBehaviorSanitizer.

Two small drivers (tests/sanitize/) are compiled with gcc / g++ -fsanitize=address,undefined together with
oracle/zipccl_oracle.c and with csrc/zipccl_host.cpp (kernel launchers replaced by stand-ins: no HIP, no GPU),
then run: round trips on exact-size buffers, ragged and empty splits, corrupt and truncated streams, the
three-peer reduce; table, size, offset, argument-check and switcher paths of the library's host code.
A sanitizer report or a failed check makes the run exit non-zero."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", "-static-libasan",
       "-g", "-O1", "-Wall", "-Wextra"]


def _build_and_run(tmp_path, compiler, sources, extra, exe):
    if shutil.which(compiler) is None:
        pytest.skip(f"{compiler} not installed")
    out = str(tmp_path / exe)
    subprocess.check_call([compiler] + SAN + extra + sources + ["-o", out, "-lm"])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([out], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-4000:]
    return r.stdout


def test_oracle_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    out = _build_and_run(tmp_path, "gcc", [os.path.join(ROOT, "oracle", "zipccl_oracle.c"),
                                           os.path.join(ROOT, "tests", "sanitize", "oracle_driver.c")],
                         ["-std=c11", "-static-libubsan"], "oracle_san")
    assert "oracle sanitizer driver: ok" in out


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    csrc = os.path.join(ROOT, "paper_2604_27844_amd", "csrc")
    out = _build_and_run(tmp_path, "g++", [os.path.join(csrc, "zipccl_host.cpp"),
                                           os.path.join(ROOT, "tests", "sanitize", "host_driver.cpp")],
                         ["-std=c++17", "-I", os.path.join(ROOT, "include"), "-I", csrc], "host_san")
    assert "host sanitizer driver: ok" in out
