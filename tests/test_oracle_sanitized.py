"""The oracle's pins once more on a build of oracle/mnnq_oracle.c with AddressSanitizer and
UndefinedBehaviorSanitizer (host code only, no GPU): an out-of-bounds index, a signed overflow or a
misaligned access in the checker itself would otherwise go unnoticed."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
PINS = ["tests/test_oracle_quantizers.py", "tests/test_oracle_linear.py", "tests/test_oracle_minfloat.py",
        "tests/test_oracle_int8.py", "tests/test_oracle_a16_minfloat.py"]


def test_pins_pass_on_the_sanitized_oracle():
    asan = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    if not os.path.isabs(asan) or not os.path.exists(asan):
        pytest.skip("no libasan for this gcc")
    env = dict(os.environ, MNNQ_ORACLE_SANITIZE="1", LD_PRELOAD=asan,
               ASAN_OPTIONS="detect_leaks=0:halt_on_error=1:abort_on_error=1",
               UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")
    r = subprocess.run([sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider"] + PINS,
                       cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, (r.stdout[-3000:], r.stderr[-3000:])
    assert " passed" in r.stdout
