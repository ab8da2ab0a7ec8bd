"""The oracle's pins once more with the oracle compiled under AddressSanitizer and
UndefinedBehaviorSanitizer (host code only: gcc, no GPU): an out-of-bounds index, a
use after free, a signed overflow or a misaligned access in the checker itself would
make every parity claim that rests on it worthless.  The sanitizer runtime has to be
the first library of the process, so the pins run in a child interpreter that preloads it."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["tests/test_oracle_attn.py", "tests/test_oracle_score.py", "tests/test_oracle_select.py",
        "tests/test_oracle_gather.py", "tests/test_oracle_accept.py", "tests/test_oracle_tree.py",
        "tests/test_oracle_baseline.py"]


def _runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_oracle_pins_under_asan_and_ubsan():
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("gcc's AddressSanitizer runtime is not installed")
    env = dict(os.environ)
    env.update({
        "SPECVLM_ORACLE_SANITIZE": "1",
        # the sanitizer runtime must come first in the list; whatever was preloaded stays behind it
        "LD_PRELOAD": ":".join(x for x in (asan, os.environ.get("LD_PRELOAD", "")) if x),
        # the interpreter's own allocations are not the subject; any error in the oracle aborts the child
        "ASAN_OPTIONS": "detect_leaks=0:abort_on_error=1:halt_on_error=1",
        "UBSAN_OPTIONS": "halt_on_error=1:print_stacktrace=1",
        "OMP_NUM_THREADS": "4",
    })
    # the slowest pin (a Monte-Carlo over 2e5 trials) is left to the plain build
    res = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *PINS,
                          "-k", "not chi_square and not monte_carlo"],
                         cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (res.stdout + res.stderr)[-3000:]
    assert res.returncode == 0, tail
    assert "passed" in res.stdout and "ERROR: AddressSanitizer" not in tail and "runtime error" not in tail, tail
