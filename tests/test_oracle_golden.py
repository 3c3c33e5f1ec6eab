"""The oracle still produces the outputs whose digests are stored under tests/golden/ (drift guard)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_oracle_outputs_match_stored_digests(orc):
    script = os.path.join(ROOT, "tests", "golden", "make_oracle_digests.py")
    r = subprocess.run([sys.executable, script, "--check"], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
