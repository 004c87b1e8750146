"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol the
header declares, and rejects bad arguments before touching the HIP runtime."""
import ctypes
import os
import re
import sys

import pytest

import paper_2209_10778_amd as nfad

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "nfad.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(nfad_[a-z_0-9]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    assert declared_functions() == sorted([
        "nfad_fwd", "nfad_bwd", "nfad_recompute_fwd", "nfad_recompute_bwd", "nfad_saveall_num_saved",
        "nfad_saveall_fwd", "nfad_saveall_bwd", "nfad_status_string", "nfad_version",
        "nfad_chain_count", "nfad_chain_name", "nfad_chain_program", "nfad_chain_fwd",
        "nfad_chain_compile", "nfad_chain_release", "nfad_chain_log", "nfad_chain_compile_multi",
        "nfad_chain_num_outputs", "nfad_chain_fwd_multi", "nfad_bwd_multi", "nfad_chain_kernel"])


def test_library_exports_every_declared_symbol():
    L = ctypes.CDLL(nfad.lib_path())
    for name in declared_functions():
        assert hasattr(L, name), f"libnfad.so does not export {name}"


def test_version_and_status_strings():
    assert nfad.nfad_version() >= 100
    seen = {nfad.nfad_status_string(s) for s in range(9)}
    assert len(seen) == 9 and all(seen)
    assert nfad.nfad_status_string(0) == "ok"
    assert nfad.nfad_status_string(12345) == "unknown status"


def test_num_saved():
    assert [nfad.nfad_saveall_num_saved(k) for k in nfad.KINDS] == [4, 3, 2, 2]
    assert nfad.nfad_saveall_num_saved(9) == -1


def test_argument_validation_precedes_any_launch():
    L = nfad.lib()
    A = 1 << 20           # fake, suitably aligned addresses: validation never dereferences them
    OK, EKIND, EDTYPE, ENULL, EALIGN, EALIAS = 0, 1, 2, 3, 4, 5
    assert L.nfad_fwd(4, A, A + 64, A + 128, 8, 0, None) == EKIND
    assert L.nfad_fwd(-1, A, A + 64, A + 128, 8, 0, None) == EKIND
    assert L.nfad_fwd(0, A, A + 64, A + 128, 8, 3, None) == EDTYPE
    assert L.nfad_fwd(0, None, A + 64, A + 128, 8, 0, None) == ENULL
    assert L.nfad_fwd(0, A, None, A + 128, 8, 0, None) == ENULL
    assert L.nfad_fwd(0, A, A + 64, None, 8, 0, None) == ENULL
    assert L.nfad_fwd(0, A + 2, A + 64, A + 128, 8, 0, None) == EALIGN    # fp32 needs 4-byte alignment
    assert L.nfad_fwd(0, A + 1, A + 64, A + 128, 8, 2, None) == EALIGN    # bf16 needs 2-byte alignment
    assert L.nfad_fwd(0, A, A + 64, A + 64, 8, 0, None) == EALIAS
    assert L.nfad_fwd(0, None, None, None, 0, 0, None) == OK               # n == 0: nothing to do
    assert L.nfad_fwd(0, None, None, None, 0, 9, None) == EDTYPE           # but dtype is still checked
    assert L.nfad_bwd(None, A, A, 4, 1, None) == ENULL
    assert L.nfad_bwd(A, A, A + 1, 4, 1, None) == EALIGN
    assert L.nfad_bwd(None, None, None, 0, 1, None) == OK
    assert L.nfad_recompute_fwd(7, A, A, 4, 0, None) == EKIND
    assert L.nfad_recompute_fwd(2, A, None, 4, 0, None) == ENULL
    assert L.nfad_recompute_bwd(2, A, None, A, 4, 0, None) == ENULL
    assert L.nfad_recompute_bwd(2, A, A, A, 4, 5, None) == EDTYPE
    vpp = ctypes.c_void_p * 4
    assert L.nfad_saveall_fwd(2, A, A + 64, None, 4, 0, None) == ENULL
    assert L.nfad_saveall_fwd(2, A, A + 64, vpp(None, None, None, None), 4, 0, None) == ENULL
    assert L.nfad_saveall_fwd(0, A, A + 64, vpp(None, A + 128, A + 192, A + 128), 4, 0, None) == EALIAS
    assert L.nfad_saveall_fwd(5, A, A + 64, vpp(A, A, A, A), 4, 0, None) == EKIND
    assert L.nfad_saveall_bwd(1, A, vpp(A, A, None, None), A, 4, 0, None) == ENULL
    assert L.nfad_saveall_bwd(1, A, None, A, 0, 0, None) == OK


def test_malformed_chain_programs_are_rejected_on_the_host():
    """Parsing precedes any compiler or HIP call, so this runs without a GPU."""
    L = nfad.lib()
    cid = ctypes.c_int(-7)
    for bad in (b"x x", b"x +", b"x foo", b"", b"1 2 +", b"x 1e999 *", b"x ; system", b"x nan *",
                b" ".join([b"x"] * 200 + [b"+"] * 199)):
        assert L.nfad_chain_compile(bad, ctypes.byref(cid)) == 7, bad
        assert cid.value == -7 and nfad.nfad_chain_log()
    assert L.nfad_chain_compile(None, ctypes.byref(cid)) == 3
    assert L.nfad_chain_compile(b"x tanh", None) == 3
    assert L.nfad_chain_release(5) == 1 and L.nfad_chain_release(1000 + 12345) == 1
    progs = (ctypes.c_char_p * 5)(b"x tanh", b"x exp", b"x x *", b"x neg", b"x sigmoid")
    assert L.nfad_chain_compile_multi(progs, 0, ctypes.byref(cid)) == 1
    assert L.nfad_chain_compile_multi(progs, 5, ctypes.byref(cid)) == 1
    bad = (ctypes.c_char_p * 2)(b"x tanh", b"x +")
    assert L.nfad_chain_compile_multi(bad, 2, ctypes.byref(cid)) == 7 and "program 1" in nfad.nfad_chain_log()
    assert nfad.nfad_chain_num_outputs(0) == 1 and nfad.nfad_chain_num_outputs(-3) == -1
    A = 1 << 20
    vpp = ctypes.c_void_p * 4
    assert L.nfad_bwd_multi(vpp(A, A, A, A), vpp(A, A, A, A), 0, A, 4, 0, None) == 1
    assert L.nfad_bwd_multi(vpp(A, A, A, A), vpp(A, A, A, A), 5, A, 4, 0, None) == 1
    assert L.nfad_bwd_multi(vpp(A, None, A, A), vpp(A, A, A, A), 2, A, 4, 0, None) == 3
    assert L.nfad_bwd_multi(None, None, 2, None, 0, 0, None) == 0
    assert L.nfad_chain_fwd_multi(0, A, vpp(A, A, A, A), vpp(A, A, A, A), 4, 0, None) == 1    # built-in id
    assert nfad.nfad_chain_name(1000) is None or isinstance(nfad.nfad_chain_name(1000), str)


def test_binding_rejects_host_tensors_and_mismatches():
    import torch
    x = torch.zeros(8)
    with pytest.raises(ValueError):
        nfad.nfad_fwd(nfad.SWISH, x, x.clone(), x.clone())
    with pytest.raises(TypeError):
        nfad.nfad_fwd(nfad.SWISH, x.double(), x.double(), x.double())


def test_missing_library_fails_loudly(monkeypatch):
    from paper_2209_10778_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "_LIB_PATH", "/nonexistent/libnfad.so")
    with pytest.raises(ImportError):
        binding.lib()


def test_product_path_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2209_10778_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".inc", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "import oracle" not in text and "from oracle" not in text, f
                assert "nfad_oracle" not in text, f
    otext = open(os.path.join(ROOT, "oracle", "__init__.py")).read() + open(os.path.join(ROOT, "oracle", "nfad_oracle.c")).read()
    assert "paper_2209_10778_amd" not in otext


def test_header_is_plain_c_and_links(tmp_path):
    """The boundary is a C ABI: the header must compile as C99 with warnings as errors, and a C
    program must link against the library and reach the host-side validation."""
    import subprocess
    src = tmp_path / "abi.c"
    src.write_text(r"""
#include "nfad.h"
#include <stdio.h>
int main(void) {
  float buf[64];   /* 256 bytes; host memory: validation never dereferences it */
  void* a = (void*)(((size_t)buf + 63) & ~(size_t)63);
  void* b = (char*)a + 64;
  void* c = (char*)a + 128;
  int ok = 1;
  ok &= nfad_fwd(99, a, b, c, 4, NFAD_F32, 0) == NFAD_EINVAL_KIND;
  ok &= nfad_fwd(NFAD_MISH, a, b, b, 4, NFAD_F32, 0) == NFAD_EALIAS;
  ok &= nfad_bwd(a, 0, c, 4, NFAD_BF16, 0) == NFAD_ENULL;
  ok &= nfad_fwd(NFAD_SWISH, 0, 0, 0, 0, NFAD_F16, 0) == NFAD_OK;
  ok &= nfad_saveall_num_saved(NFAD_GELU_TANH) == NFAD_MAX_SAVED;
  ok &= nfad_chain_count() > 0 && nfad_chain_name(0) != 0 && nfad_chain_program(0) != 0;
  ok &= nfad_version() >= 100;
  printf("%s\n", nfad_status_string(NFAD_EALIGN));
  return ok ? 0 : 1;
}
""")
    exe = tmp_path / "abi"
    libdir = os.path.dirname(nfad.lib_path())
    subprocess.run(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-lnfad", f"-Wl,-rpath,{libdir}",
                    "-Wl,-rpath,/opt/rocm/lib"], check=True)
    r = subprocess.run([str(exe)], capture_output=True, text=True)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "aligned" in r.stdout


def test_the_plain_c_test_program_builds():
    """tests/c_abi/nfad_c_check.c (run by the GPU suite) compiles as C99 with -Werror and links
    against the library, the oracle and the HIP runtime's C API."""
    sys.path.insert(0, os.path.join(ROOT, "tests", "c_abi"))
    import build_check
    import oracle
    oracle.build()
    assert os.path.exists(build_check.build())
