"""bench.py argument handling that needs no GPU."""
import os
import subprocess
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _bench(*args):
    return subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), *args], capture_output=True, text=True,
                          timeout=120)


def test_more_than_one_gpu_is_refused_with_a_message():
    r = _bench("--gpus", "2")
    assert r.returncode == 2
    assert "one GPU only" in r.stderr and r.stdout.strip() == ""


def test_window_needs_the_fused_route():
    import torch
    if torch.cuda.is_available():
        r = _bench("--window", "10", "--decode-route", "separate", "--workload", "tiny", "--no-cpu-baseline")
        assert r.returncode == 2 and "fused decode route only" in r.stderr
    else:
        r = _bench("--window", "10", "--decode-route", "separate")
        assert r.returncode == 2 and r.stdout.strip() == ""      # refused before any GPU work either way
