"""The CPU-side native code under AddressSanitizer and UndefinedBehaviorSanitizer (host code only).

The C oracle and the host worker are compiled once more with -fsanitize=address,undefined, and the
tests that pin the oracle and check the host worker against it run again, in a child interpreter,
on those builds: an out-of-bounds read of a padded list, a misaligned vector load or a signed
overflow in an index that the plain builds survive by luck stops the run here.
"""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SAN = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-g"]
PINS = ["tests/test_oracle_digest_score.py", "tests/test_oracle_select_recall.py", "tests/test_oracle_attention_merge.py",
        "tests/test_oracle_append.py", "tests/test_golden.py", "tests/test_host_worker.py"]


def _runtime(compiler):
    path = subprocess.run([compiler, "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_and_host_worker_pins_under_asan_ubsan(tmp_path):
    asan = _runtime("gcc")
    if asan is None:
        pytest.skip("this toolchain ships no AddressSanitizer runtime")
    olib, hlib = str(tmp_path / "libscout_oracle_san.so"), str(tmp_path / "libscout_host_san.so")
    subprocess.run(["gcc", "-O1", "-std=c99", "-fPIC", "-shared", "-Wall", "-Wextra", *SAN, "-o", olib,
                    os.path.join(ROOT, "oracle", "scout_oracle.c"), "-lm"], check=True)
    subprocess.run(["g++", "-O1", "-std=c++17", "-fPIC", "-shared", "-pthread", "-Wall", "-Wextra", "-Wno-psabi", *SAN,
                    "-I", os.path.join(ROOT, "include"), "-o", hlib,
                    os.path.join(ROOT, "paper_2603_27138_amd", "csrc", "host_worker.cpp")], check=True)
    env = dict(os.environ)
    # the sanitizer runtime has to be loaded before the interpreter's own libraries; whatever is
    # preloaded already stays, behind it
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter's own allocations are never freed at exit: leak reports say nothing about our code
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1"
    env["SCOUT_ORACLE_LIB"], env["SCOUT_HOST_LIB"] = olib, hlib
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-m", "not gpu", "-p", "no:cacheprovider", *PINS], cwd=ROOT, env=env,
                         capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-4000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
