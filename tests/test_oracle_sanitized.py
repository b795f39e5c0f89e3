"""The oracle's C source under AddressSanitizer and UndefinedBehaviorSanitizer: the pins of
tests/test_oracle_backward.py and tests/test_oracle_adamw.py are run again, in a child process,
against a sanitized build of tf_oracle.c.  An out-of-bounds index, a use of uninitialised
stack, a signed overflow or a misaligned access in the oracle ends that process with an error."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _runtime(name):
    out = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return out if os.path.isabs(out) and os.path.exists(out) else None


def test_oracle_pins_hold_under_address_and_undefined_behaviour_sanitizers():
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("gcc has no AddressSanitizer runtime here")
    env = dict(os.environ)
    env["TF_ORACLE_SANITIZE"] = "1"
    # the sanitizer runtime has to be loaded before the interpreter's own libraries
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    env["OMP_NUM_THREADS"] = "4"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
           os.path.join(ROOT, "tests", "test_oracle_backward.py"), os.path.join(ROOT, "tests", "test_oracle_adamw.py")]
    res = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
    assert os.path.exists(os.path.join(ROOT, "oracle", "libtf_oracle_san.so"))
