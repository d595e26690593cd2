"""The CPU checker under AddressSanitizer + UndefinedBehaviorSanitizer (host code only, no GPU): its pins are
run once more in a child process against a sanitized build of oracle/cbd_oracle.c.  Any out-of-bounds access,
use after free, signed overflow or misaligned access in the checker aborts the child."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def sanitizer_runtime():
    out = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


@pytest.mark.timeout(900)
def test_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    rt = sanitizer_runtime()
    if rt is None:
        pytest.skip("gcc has no AddressSanitizer runtime here")
    env = dict(os.environ)
    # the sanitizer's runtime has to be loaded before the interpreter's own libraries
    env["LD_PRELOAD"] = rt + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["CBD_ORACLE_SANITIZE"] = "1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", "-m", "not gpu",
           os.path.join(ROOT, "tests", "test_oracle_pins.py")]
    r = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True)
    tail = (r.stdout + r.stderr)[-3000:]
    assert r.returncode == 0, "pins failed under the sanitizers:\n" + tail
    assert "passed" in r.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
