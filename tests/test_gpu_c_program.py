"""GPU: the boundary used from plain C.  tests/c_abi_check.c allocates with the HIP runtime's C
API, runs a DoubleSqueeze step through include/ds.h (no Python, no torch in the process) for the
1-bit and the top-k compressor and compares everything with the oracle it links."""
import os
import subprocess

import pytest

import build_c_abi_check

pytestmark = pytest.mark.gpu


def test_c_program_on_the_c_abi(gpu_device):
    binary = build_c_abi_check.build(force=False)
    r = subprocess.run([binary], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.count("equal to the oracle") == 2
