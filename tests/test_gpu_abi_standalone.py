"""The C ABI without Python or PyTorch around it: a plain HIP program
(tests/host/abi_standalone.cpp, built by __graft_entry__.build()) allocates with
hipMalloc, runs every device entry point on the default stream and on a stream
of its own, and compares every element with the CPU checker's C functions."""
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "host", "abi_standalone")


def test_c_abi_from_a_plain_hip_program():
    print("\n[gpu-case] abi_standalone", file=sys.stderr, flush=True)
    assert os.path.exists(EXE), "tests/host/abi_standalone is not built; run __graft_entry__.build()"
    out = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    assert out.stdout.startswith("ok"), out.stdout + out.stderr
