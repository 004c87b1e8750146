"""The table of run-time compiled chains on the host: a plain C++ program drives
csrc/nfad_chain_table.hpp with a stand-in kernel type (no GPU): slots are reused, the capacity
counts live chains only, chains that differ in constants share a kernel, a kernel dies with its
last user, and concurrent compile / use / release is safe."""
import os
import subprocess
import tempfile

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_chain_table_slot_reuse_sharing_and_capacity():
    src = os.path.join(ROOT, "tests", "host", "chain_table_check.cpp")
    with tempfile.TemporaryDirectory() as tmp:
        exe = os.path.join(tmp, "chain_table_check")
        subprocess.run(["g++", "-std=c++17", "-O1", "-Wall", "-Werror", "-pthread", src, "-o", exe], check=True)
        r = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0 and "all checks passed" in r.stdout, r.stdout + r.stderr


def test_table_capacity_is_checked_before_compiling_and_programs_are_parsed_on_the_host():
    """With the capacity hook at its minimum the translation errors still come first (host only),
    and a well-formed program on a machine without a GPU fails at loading, not at parsing."""
    import ctypes
    import paper_2209_10778_amd as nfad
    L = nfad.lib()
    cid = ctypes.c_int(-1)
    for prog, why in (("x 0 /", "division by the constant 0"), ("1 2 +", "does not use x"),
                      ("x +", "lacks operands"), ("x x", "leaves 2 values"), ("x foo", "unknown token"),
                      (" ".join(["x"] + [f"{1.5 + i} *" for i in range(25)]), "more than 24 constants")):
        assert L.nfad_chain_compile(prog.encode(), ctypes.byref(cid)) == 7, prog      # NFAD_EPROGRAM
        assert why in nfad.nfad_chain_log(), (prog, nfad.nfad_chain_log())
    assert nfad.nfad_chain_kernel(0) == -1 and nfad.nfad_chain_kernel(1000) == -1      # built-in, dead
