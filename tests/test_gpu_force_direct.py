"""SWCONV_FORCE_DIRECT=1 sends every entry point to its one-thread-per-output kernel.  The switch is read once
per process, so the cases run in a child process (tests/force_direct_child.py), which checks both the parity
bars and, through sw_last_kernel(), that a direct kernel is what ran."""
import os
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.mark.gpu
def test_every_entry_point_on_its_direct_kernel():
    env = dict(os.environ, SWCONV_FORCE_DIRECT="1")
    p = subprocess.run([sys.executable, "-u", os.path.join(ROOT, "tests", "force_direct_child.py")], env=env,
                       capture_output=True, text=True, timeout=110)
    assert p.returncode == 0, p.stdout[-3000:] + p.stderr[-3000:]
    assert p.stdout.strip().endswith("force-direct ok")
