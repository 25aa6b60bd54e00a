"""The C ABI called from C: tests/c_abi_caller.c (C99, HIP runtime C API, no Python, no C++) runs a
self-attention and a masked cross-attention through include/dit_attn.h and compares them with the
C oracle linked into the same program.  The binary is built beforehand by
`python tests/build_c_caller.py` (or __graft_entry__.build())."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu

EXE = os.path.join(os.path.dirname(os.path.abspath(__file__)), "bin", "c_abi_caller")


def test_c_program_calls_the_library_and_matches_the_oracle():
    if not os.path.exists(EXE):
        pytest.skip("tests/bin/c_abi_caller is not built (python tests/build_c_caller.py)")
    r = subprocess.run([EXE], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, timeout=120)
    print(r.stdout)
    assert r.returncode == 0, r.stdout
    assert "c caller ok" in r.stdout
