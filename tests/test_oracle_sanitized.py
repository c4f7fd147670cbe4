"""The CPU checker under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU): the pins of the
checker are run once more in a child process against a build of oracle/grf_oracle.c with -fsanitize=address,undefined.
The checker indexes with caller-supplied CSR arrays everywhere; any access outside an array or undefined operation
aborts the child with a report."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_checker_pins_under_address_and_undefined_behaviour_sanitizers():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("gcc's libasan.so is not installed")
    env = dict(os.environ)
    env["GRF_ORACLE_SANITIZE"] = "1"
    env["ASAN_OPTIONS"] = "detect_leaks=0"          # the interpreter's own allocations are not the subject
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    pins = ["tests/test_oracle_pins.py", "tests/test_oracle_backward_pins.py", "tests/test_oracle_knn_pins.py"]
    run = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *pins], cwd=ROOT, env=env,
                         capture_output=True, text=True, timeout=900)
    text = run.stdout + run.stderr
    assert run.returncode == 0, text[-3000:]
    assert "AddressSanitizer" not in text and "runtime error" not in text, text[-3000:]
    assert os.path.exists(os.path.join(ROOT, "oracle", "libgrf_oracle_san.so"))      # the sanitized build is what ran
