"""The oracle's pins once more under AddressSanitizer and UndefinedBehaviorSanitizer (host code only): the C source is
built with -fsanitize=address,undefined -fno-sanitize-recover=all and the oracle test files run in a child interpreter
that has the ASan runtime preloaded.  Any out-of-bounds access, overflow or misaligned access in the oracle ends the
child with an error."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PIN_FILES = ["tests/test_oracle_prefill.py", "tests/test_oracle_decode.py", "tests/test_oracle_query.py",
             "tests/test_oracle_retention.py"]


def test_oracle_pins_pass_under_address_and_undefined_behaviour_sanitizers():
    try:
        libasan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    except (OSError, subprocess.CalledProcessError):
        pytest.skip("no gcc")
    if not os.path.isabs(libasan) or not os.path.exists(libasan):
        pytest.skip("no ASan runtime beside gcc")
    env = dict(os.environ)
    env["SKVO_SANITIZE"] = "1"
    env["LD_PRELOAD"] = libasan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    env["ASAN_OPTIONS"] = "detect_leaks=0:halt_on_error=1"          # the interpreter itself leaks by design
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    probe = subprocess.run([sys.executable, "-c", "import numpy, ctypes; print('ok')"], env=env, capture_output=True, text=True,
                           cwd=ROOT)
    if probe.returncode != 0 or "ok" not in probe.stdout:
        pytest.skip("this interpreter does not start with the ASan runtime preloaded: " + probe.stderr[-300:])
    run = subprocess.run([sys.executable, "-m", "pytest", *PIN_FILES, "-x", "-q", "-p", "no:cacheprovider"], env=env,
                         capture_output=True, text=True, cwd=ROOT, timeout=900)
    tail = (run.stdout + run.stderr)[-3000:]
    assert run.returncode == 0, tail
    assert "passed" in run.stdout and "AddressSanitizer" not in tail and "runtime error" not in tail, tail
