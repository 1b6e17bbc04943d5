"""The oracle's pins once more, with the oracle compiled under AddressSanitizer + UndefinedBehaviorSanitizer
(host code only, no GPU): an out-of-bounds index or an overflow in the checker would otherwise go unnoticed
as long as the numbers come out right."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_pins_pass_under_address_and_ub_sanitizers():
    if os.environ.get("PROBE_ORACLE_SANITIZE") == "1":
        pytest.skip("already inside the sanitized run")
    r = subprocess.run([sys.executable, os.path.join(ROOT, "oracle", "run_sanitized.py")], capture_output=True,
                       text=True, timeout=900)
    if r.returncode == 3:
        pytest.skip("no sanitizer runtime with this gcc")
    assert r.returncode == 0, (r.stdout[-3000:] + r.stderr[-3000:])
    assert " passed" in r.stdout
