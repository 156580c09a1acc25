"""The CPU oracle under AddressSanitizer and UndefinedBehaviorSanitizer: oracle/selfcheck.c drives every entry
point on small inputs; any report (out-of-bounds access, leak, signed overflow, misaligned access) fails the run."""
import os
import subprocess

from oracle import build_oracle


def test_oracle_entry_points_are_clean_under_address_and_undefined_behaviour_sanitizers():
    exe = build_oracle.build_selfcheck()
    r = subprocess.run([exe], capture_output=True, text=True, env=dict(os.environ, OMP_NUM_THREADS="2"), timeout=300)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "oracle selfcheck ok" in r.stdout
