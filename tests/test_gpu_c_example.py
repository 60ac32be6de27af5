"""The boundary is a C ABI: a plain C program (gcc, no Python, no torch) links the library, runs a ring
all-reduce with a channel failure and checks every rank against the exact sum."""
import os
import subprocess

import pytest

from gpu_util import say

pytestmark = pytest.mark.gpu

HERE = os.path.dirname(os.path.abspath(__file__))
EXE = os.path.join(os.path.dirname(HERE), "paper_2512_25059_amd", "examples", "ring_allreduce")


def test_c_program_runs_the_ring():
    assert os.path.exists(EXE), "the example is built by paper_2512_25059_amd.build.build()"
    say("C example: ring_allreduce")
    res = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    assert res.returncode == 0, res.stdout + res.stderr
    assert "every rank holds the exact sum" in res.stdout
    # 1 MiB chunk, weights 2:2:1:1 with channel 1 down: shares 2/4, 0, 1/4, 1/4 in units of 256 bytes
    assert "chunk of 1048576 bytes over channels: 524288 0 262144 262144" in res.stdout
