"""The C oracle under AddressSanitizer + UndefinedBehaviorSanitizer: the pin tests, the generator tests and the
host-side argument checks of the library once more in a child process that loads the sanitized build of
oracle/plx_oracle.c.  Any out-of-bounds access, use of uninitialised indices that leave an array, signed overflow
or misaligned access in the oracle's loops ends the child with a report and fails this test.  CPU only."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_under_asan_and_ubsan():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no AddressSanitizer runtime next to gcc")
    env = dict(os.environ)
    env["PLX_ORACLE_SANITIZE"] = "1"
    # the sanitizer runtime has to be loaded before the interpreter's own libraries; a preload that is already set stays
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # the interpreter and numpy are not instrumented: their own leaks and link order are not this test's subject
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=99"
    env["UBSAN_OPTIONS"] = "print_stacktrace=1:halt_on_error=1:exitcode=98"
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
                        os.path.join(ROOT, "tests", "test_oracle_pins.py")], cwd=ROOT, env=env, capture_output=True, text=True,
                       timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert "passed" in r.stdout and "libplx_oracle_san.so" in subprocess.run(
        ["ls", os.path.join(ROOT, "oracle")], capture_output=True, text=True).stdout, tail
