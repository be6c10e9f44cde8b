"""The C ABI used from plain C, with no Python and no torch in the process: tests/abi_step.c
runs one small step with a failed rank through include/eep.h on buffers from hipMalloc and
compares every result with the C oracle itself.  The binary is built by build()
(tests/abi_step_build.py) from the two libraries that are already there."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
BIN = os.path.join(HERE, "abi_step.bin")


def test_one_step_from_plain_c_matches_the_oracle():
    if not os.path.exists(BIN):      # normally built by build(); a one-second gcc link otherwise
        import runpy
        runpy.run_path(os.path.join(HERE, "abi_step_build.py"))["build"]()
    done = subprocess.run([BIN], capture_output=True, text=True, timeout=120)
    assert done.returncode == 0, done.stdout[-2000:] + done.stderr[-2000:]
    assert "abi_step ok: N = 256 rows, rank 2 got 0" in done.stdout
