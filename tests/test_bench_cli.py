"""Command line of bench.py that needs no GPU: more than one GPU is refused with a message before anything
touches the device (every figure of this build is one GPU's)."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_more_than_one_gpu_is_refused_with_a_message():
    for n in ("2", "8"):
        r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", n, "--steps", "1", "--warmup", "0"],
                           capture_output=True, text=True, timeout=120)
        assert r.returncode != 0
        assert "ONE GPU" in (r.stdout + r.stderr) and "--gpus " + n in (r.stdout + r.stderr)
        assert not r.stdout.strip().startswith("{")          # no benchmark line


def test_help_lists_the_modes():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--help"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0
    for word in ("--gpus", "--steps", "--warmup", "--mode", "prefill", "batched", "generate", "backward"):
        assert word in r.stdout
