"""Runs the plain C program tests/c_abi_demo.c (built by
__graft_entry__.build()) on the GPU: the C ABI used without Python or PyTorch,
checked against the oracle compiled into the program."""
import os
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
EXE = os.path.join(HERE, "_build", "c_abi_demo")


@pytest.mark.gpu
def test_c_program_drives_the_library():
    assert os.path.exists(EXE), "tests/_build/c_abi_demo is not built; run __graft_entry__.build()"
    print("case: C ABI demo", flush=True)
    r = subprocess.run([EXE], capture_output=True, text=True, timeout=120)
    print(r.stdout, r.stderr)
    assert r.returncode == 0 and "OK, K = 3," in r.stdout and "OK, K = 9," in r.stdout
