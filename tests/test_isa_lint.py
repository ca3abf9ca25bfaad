"""The hand-scheduled loads of pointwise_ring_kernel survive the compiler (no GPU needed).

Compiles the kernels to gfx950 assembly and runs the check that ships beside the kernel source:
no instruction may touch a register that an asm-issued load is still filling."""
import os
import shutil
import subprocess
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
SCRIPT = os.path.join(ROOT, "paper_2012_00596_amd", "csrc", "check_async_loads.py")


@pytest.mark.skipif(shutil.which("hipcc") is None, reason="hipcc not on PATH")
def test_async_loads_are_not_touched_before_their_wait():
    r = subprocess.run([sys.executable, SCRIPT], capture_output=True, text=True, timeout=900)
    assert r.returncode == 0, r.stdout + r.stderr
