"""The C ABI from a plain C99 program (tests/c_abi/nfad_c_check.c): no Python and no PyTorch
between the caller and libnfad.  The program allocates with the HIP runtime's C API, calls all
six passes for the four activations plus a run-time compiled chain, and checks the results
against the fp64 oracle it links; this test only runs it and reads its exit status."""
import os
import subprocess

import pytest

pytestmark = pytest.mark.gpu
BINARY = os.path.join(os.path.dirname(os.path.abspath(__file__)), "c_abi", "nfad_c_check")


def test_plain_c_program_passes_all_checks():
    assert os.path.exists(BINARY), f"{BINARY} is missing: run __graft_entry__.build() (or tests/c_abi/build_check.py)"
    r = subprocess.run([BINARY], capture_output=True, text=True, timeout=120)
    print(r.stdout)
    print(r.stderr)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-2000:]
    assert "all checks passed" in r.stdout
