"""The C ABI from a plain C program (no Python, no PyTorch in the process): tests/cabi/cabi_check.c,
compiled beforehand by tests/cabi/build_cabi.py (__graft_entry__.build() runs it)."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cabi", "cabi_check")


def test_plain_c_program_gets_the_oracles_bytes():
    assert os.path.exists(EXE), "run python tests/cabi/build_cabi.py (or __graft_entry__.build()) first"
    out = subprocess.run([EXE], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=100)
    print(out.stdout, flush=True)
    assert out.returncode == 0 and "cabi ok" in out.stdout, out.stdout
