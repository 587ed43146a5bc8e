"""The C ABI used from a plain host program (HIP runtime + include/dsk.h, no Python objects, no
torch): the example builds its own inputs, runs the compression pass and a decode step, and checks
the attention output against a double-precision softmax it computes itself."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

EXE = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "paper_2602_03184_amd", "dsk_example")


def test_host_only_example_runs_and_checks_itself():
    assert os.path.exists(EXE), "build first: python paper_2602_03184_amd/build.py"
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "dsk_example: ok" in r.stdout
    print(r.stdout.strip())
