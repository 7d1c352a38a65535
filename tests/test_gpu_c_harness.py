"""The library called from a plain C program (no Python, no torch): GPU parity with the
oracle and the buffer checks at exact allocation extents.  See tests/c_harness/."""
import os
import subprocess
import sys

import pytest

sys.path.insert(0, os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_harness"))
import build_harness  # noqa: E402

pytestmark = pytest.mark.gpu


def test_c_program_matches_the_oracle_and_refuses_bad_buffers():
    exe = build_harness.EXE
    if not os.path.exists(exe):
        exe = build_harness.build()
    p = subprocess.run([exe], capture_output=True, text=True, timeout=100)
    sys.stdout.write(p.stdout)
    sys.stderr.write(p.stderr)
    assert p.returncode == 0, p.stdout + p.stderr
    assert "c parity ok" in p.stdout
    assert "FAILED" not in p.stdout
