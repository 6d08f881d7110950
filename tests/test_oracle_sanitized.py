"""The oracle's pins once more with the oracle compiled under AddressSanitizer and UndefinedBehaviorSanitizer
(host code only): an out-of-bounds index, a use of uninitialised stack or heap bounds, a signed overflow or a
misaligned access anywhere in the oracle's C code aborts the child process.  Runs on the CPU."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    path = subprocess.check_output(["gcc", f"-print-file-name={name}"], text=True).strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


@pytest.mark.skipif(os.environ.get("QSAC_ORACLE_SANITIZE") == "1", reason="already inside the sanitized run")
def test_oracle_pins_pass_under_asan_and_ubsan():
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("no AddressSanitizer runtime beside gcc")
    env = dict(os.environ)
    env.update({
        "QSAC_ORACLE_SANITIZE": "1",
        "LD_PRELOAD": asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else ""),
        # the interpreter itself is not instrumented: its own allocations are not this test's business
        "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=1:verify_asan_link_order=0",
        "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1",
        "OMP_NUM_THREADS": "4",
    })
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
           os.path.join(ROOT, "tests", "test_oracle_pins.py"), os.path.join(ROOT, "tests", "test_oracle_step.py")]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, tail
    assert " passed" in r.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
