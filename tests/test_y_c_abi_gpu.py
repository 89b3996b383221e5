"""The library called from a C++ program through include/fef.h alone (no Python, no torch in that
process): identical draft and target states accept the whole window, repeated calls give the same
bits, a short workspace is refused.  The program is built with the library."""
import os
import subprocess

import pytest

from paper_2605_14305_amd.build import HARNESS

pytestmark = pytest.mark.gpu


def test_c_program_through_the_header():
    if not os.path.exists(HARNESS):
        raise RuntimeError(f"{HARNESS} is missing: run `python -m paper_2605_14305_amd.build`")
    r = subprocess.run([HARNESS], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr, flush=True)
    assert r.returncode == 0 and r.stdout.strip().endswith("OK")
