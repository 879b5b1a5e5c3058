"""The C oracle built with AddressSanitizer and UndefinedBehaviorSanitizer must pass its pins without a report:
an index one past a row, a read of an uninitialised bound or a signed overflow in the plain loops would otherwise go
unnoticed as long as the numbers come out right.  CPU only; runs the pin files in a child process that has the
sanitizer's runtime preloaded (it has to be the first library of the process)."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_on_a_sanitizer_build():
    asan = subprocess.check_output(["gcc", "-print-file-name=libasan.so"], text=True).strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("this gcc ships no libasan.so")
    env = dict(os.environ)
    env["GCN_ORACLE_SANITIZE"] = "1"
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1:abort_on_error=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "tests/test_oracle_pins.py",
           "tests/test_tile_reference.py"]
    r = subprocess.run(cmd, cwd=ROOT, env=env, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=900)
    if "ASan runtime does not come first" in r.stdout:
        pytest.skip("another preloaded library comes before the sanitizer's runtime on this machine")
    assert r.returncode == 0, r.stdout[-4000:]
    assert "ERROR: AddressSanitizer" not in r.stdout and "runtime error:" not in r.stdout, r.stdout[-4000:]
    assert " passed" in r.stdout
