"""The oracle under the host sanitizers (CPU only; nothing here touches a GPU or the HIP library).

1. UndefinedBehaviorSanitizer: a copy of the oracle built with -fsanitize=undefined (any finding aborts) is
   loaded in place of the regular build and ALL pin tests run against it.
2. AddressSanitizer + UndefinedBehaviorSanitizer: tests/oracle_sanitizer_driver.cpp includes the oracle's
   source and walks every entry point over the shapes the parity tests use, as one instrumented program."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SRC = os.path.join(ROOT, "oracle", "mpe_oracle.cpp")
PINS = ["tests/test_oracle_pins.py", "tests/test_oracle_tag_pins.py", "tests/test_oracle_gru_pins.py"]


def _compiles(flags):
    r = subprocess.run(["g++", "-x", "c++", "-", "-o", os.devnull] + flags, input="int main(){return 0;}", text=True,
                       capture_output=True)
    return r.returncode == 0


def test_pins_pass_on_an_oracle_built_with_ubsan(tmp_path):
    flags = ["-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
    if not _compiles(flags):
        pytest.skip("this g++ has no UndefinedBehaviorSanitizer runtime")
    lib = str(tmp_path / "liboracle_ubsan.so")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-fPIC", "-shared", "-pthread"] + flags +
                          ["-o", lib, SRC])
    env = dict(os.environ, MPE_ORACLE_LIB=lib, UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    r = subprocess.run([sys.executable, "-m", "pytest"] + PINS + ["-x", "-q", "-s", "-m", "not gpu", "-p", "no:cacheprovider"],
                       cwd=ROOT, env=env, capture_output=True, text=True)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "runtime error" not in r.stderr


def test_every_entry_point_is_clean_under_asan_and_ubsan(tmp_path):
    flags = ["-fsanitize=address,undefined", "-fno-sanitize-recover=all", "-static-libasan"]
    if not _compiles(flags):
        pytest.skip("this g++ has no AddressSanitizer runtime")
    exe = str(tmp_path / "oracle_sanitizer_driver")
    subprocess.check_call(["g++", "-std=c++17", "-O1", "-g", "-ffp-contract=off", "-pthread"] + flags +
                          ["-o", exe, os.path.join(ROOT, "tests", "oracle_sanitizer_driver.cpp")])
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=600)
    assert r.returncode == 0, (r.stdout + r.stderr)[-3000:]
    assert "oracle sanitizer driver: ok" in r.stdout and "ERROR" not in r.stderr
