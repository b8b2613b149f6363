"""The library driven from a program written in plain C (tests/c_abi_demo.c): no Python, no torch."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_plain_c_program_runs_the_path(gpu_device):
    sys.path.insert(0, ROOT)
    import __graft_entry__ as entry
    exe = os.path.join(ROOT, "paper_2406_12335_amd", "_build", "c_abi_demo")
    if not os.path.exists(exe):
        exe = entry.build_c_demo()
    print("[case] %s" % exe, flush=True)
    res = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "c_abi_demo ok" in res.stdout
